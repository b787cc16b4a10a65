// Step 2 on the matrix cores, head_dim 128, bf16: both passes of the query-driven
// score with the keys streamed through LDS by direct global->LDS loads.
// (Paper: Algorithm 1 first stage, alpha_l = Softmax(Q_s K'^T / sqrt(d_k)) over the
// context keys; Sec. 4.2 mean over the user-query tokens; Appendix E mean over heads.)
//
// A workgroup of 8 waves (two per SIMD, so that the softmax arithmetic of one wave runs
// under the matrix instructions and waits of the other) owns 256 columns (query token,
// head of one kv group) and one split of the key range; a wave owns 32 of them.  The
// columns are the ROWS of the MFMA tile here,
//     S [32 cols x 32 keys] = Q (A operand, registers) x K^T (B operand, LDS)
// so that a lane holds one key (l % 32) of a 32-key block and, in its 16
// accumulator registers, 16 of the 32 columns.  Sums over keys (pass 1: the
// normaliser of a column) and sums over columns (pass 2: the score of a key) are
// then both plain register additions in the hot loop; lanes meet only at the end
// of the kernel (pass 1) or once per 64-key tile through one permlane swap (pass 2).
//
//   pass 1  per column: (reference maximum, sum of exp2((s - ref) c)) over the
//           split.  The reference of a lane's column is fixed by the first tile and
//           is raised only when a tile's probabilities leave the safe range, which is
//           detected from their sum (no maximum in the hot loop).
//   pass 2  per key: sum over the workgroup's columns of exp2(s c - lse2[col]);
//           waves w and w + 4 add their sums through LDS and one partial per (workgroup
//           column block, wave pair) goes to memory; finish_score_kernel adds the
//           partials of a key in a fixed order, so the score is deterministic.
//
// K tiles of 64 keys go through a 6-stage LDS ring (16 KB per stage), requested five
// tiles ahead; layout and 16-byte-chunk XOR swizzle are those of the attention
// kernel.  One softmax step (two scores) follows every MFMA; each MFMA's key operand
// is read from LDS six MFMAs before it, into a ring of eight registers quadruples.
#include <atomic>

#include "score_common.h"

namespace pkv {

namespace {

constexpr int D = 128;
constexpr int KC = D / 16;
constexpr int kTile = 64;                   // keys per LDS stage
constexpr int NS = 6;
constexpr int kStage = kTile * D * 2;       // 16 KB
constexpr int kLdsBytes = NS * kStage;

__device__ __forceinline__ void dma16(const void* gbase, uint32_t voffset, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2"
        :
        : "s"(lds_base), "v"(voffset), "s"(gbase)
        : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

constexpr int kScoreWaves = 8;

template <int PASS, int NW>
__global__ __launch_bounds__(64 * NW) void score_dma128_kernel(ScoreParams p) {
    static_assert(NW == 8, "256 columns over 8 waves of 32 (the operand ring below assumes it)");
    static_assert(NS == 6, "the main loop is unrolled once round the ring");
    constexpr int NCB = 8 / NW;      // 32-column blocks of a wave
    constexpr int FILLS = 16 / NW;   // fill instructions of a wave per tile (4 key rows each)
    extern __shared__ __align__(16) unsigned char smem[];
    // pass 2 with 8 waves: waves w and w + 4 add their key sums before they leave the CU
    __shared__ float s_pair[2][4][kTile];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5, l32 = lane & 31;

    // kv head fastest: the workgroups that stream the same K slice share an XCD's L2
    int wg = blockIdx.x;
    const int g = wg % p.hkv;
    wg /= p.hkv;
    const int split = wg % p.n_splits;
    const int cblk = wg / p.n_splits;
    const int key_begin = split * p.split_len;
    const int key_end = min(p.n_ctx, key_begin + p.split_len);
    const int n_iter = __builtin_amdgcn_readfirstlane((key_end - key_begin + kTile - 1) / kTile);
    if (n_iter <= 0) return;   // block-uniform (cannot happen with the launcher's plan)
    const int ncol_g = p.nq * p.group;
    const float c2 = p.scale_log2;

    // ---- Q as A operands: row l32 of column block cb ------------------------------------
    bf16x8 qreg[NCB][KC];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        const int col = cblk * 256 + wave * (32 * NCB) + cb * 32 + l32;
        const bool valid = col < ncol_g;
        const int qi = valid ? col / p.group : 0;
        const int h = g * p.group + (valid ? col % p.group : 0);
        const bf16_t* qp = p.q + ((int64_t)qi * p.hq + h) * D + hh * 8;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            if (valid) {
                qreg[cb][kc] = *reinterpret_cast<const bf16x8*>(qp + kc * 16);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) qreg[cb][kc][e] = (bf16_t)0.0f;
            }
        }
    }
    // accumulator register r of column block cb belongs to this column:
    auto acc_col = [&](int cb, int r) {
        return cblk * 256 + wave * (32 * NCB) + cb * 32 + 8 * (r / 4) + 4 * hh + (r % 4);
    };

    // ---- global -> LDS: wave w fills key rows (64/NW) w .. (64/NW) (w+1) - 1 of every stage --
    const uint32_t k_row_bytes = (uint32_t)p.hkv * D * 2;
    int krow[FILLS];
    uint32_t kchunk16[FILLS];
#pragma unroll
    for (int i = 0; i < FILLS; ++i) {
        const int r = 4 * FILLS * wave + 4 * i + (lane >> 4);
        krow[i] = r;
        kchunk16[i] = (uint32_t)(((lane & 15) ^ (r & 15)) * 16);
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds0 + wave * 4 * FILLS * 256);
    const bf16_t* const k_head = p.k + (int64_t)g * D;
    // tile T of the split (clamped to its last tile) into ring slot T % NS
    auto dma_tile = [&](int T) {
        const int slot = T % NS;
        const int t = min(T, n_iter - 1);
        const int t0 = key_begin + t * kTile;
        const bf16_t* gb = k_head + (int64_t)t0 * p.hkv * D;
        const int last = p.n_ctx - 1 - t0;   // rows past the context re-read its last key
#pragma unroll
        for (int i = 0; i < FILLS; ++i)
            dma16(gb, (uint32_t)min(krow[i], last) * k_row_bytes + kchunk16[i],
                  lds_wave + slot * kStage + i * 1024);
    };

    // ---- LDS -> B operands: key l32 of block kb, contraction chunk kc ------------------------
    uint32_t kaddr[KC];
    {
        const uint32_t a0 = l32 * 256 + (((l32 & 15) ^ hh) * 16);
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) kaddr[kc] = a0 ^ (kc << 5);
    }
    // The B operands of a tile are used once each (16 MFMAs: contraction chunk kc = i / 2,
    // key block kb = i % 2), so they pass through a ring of 8 registers quadruples, read from
    // LDS kLook MFMAs before their use.
    constexpr int kLook = 6;
    bf16x8 kq[8];
    // STAGE = the ring stage of tile T when the caller knows it at compile time (the main loop
    // is unrolled over the ring), else -1.  With a known stage the whole offset fits the
    // 16-bit immediate of the LDS instruction - from a second copy of the lane addresses,
    // 64 KB on, for stages 4 and 5 - and no address arithmetic is left in the loop.
    uint32_t kaddr_hi[KC];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) kaddr_hi[kc] = kaddr[kc] + 4 * kStage;
    auto load_op = [&](int T, int STAGE, int i, int slot) {
        const unsigned char* a;
        if (STAGE < 0) a = smem + (T % NS) * kStage + kaddr[i >> 1];
        else if (STAGE < 4) a = smem + STAGE * kStage + kaddr[i >> 1];
        else a = smem + (STAGE - 4) * kStage + kaddr_hi[i >> 1];
        kq[slot] = *reinterpret_cast<const bf16x8*>(a + (i & 1) * 32 * 256);
    };

    // ---- per-pass state --------------------------------------------------------------------
    float norm[NCB][16];  // pass 2: log2-domain normaliser of my columns (inf = no column)
    float msc[NCB][16];   // pass 1: reference maximum of my columns over this lane's keys, times c2
    float lsum[NCB][16];  //         sum of exp2(s c2 - msc) over this lane's keys, up to the
    float tsum[NCB][16];  //         previous tile; the previous tile's own sum (not yet added)
    float ksum[2] = {0.f, 0.f};   // pass 2: this tile's two keys, summed over my columns
    float pend[2] = {0.f, 0.f};   // pass 2, 8 waves: the previous tile's sums, not yet stored
    int pend_t0 = -1;
    constexpr float kGrow = 1.0e24f;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int col = acc_col(cb, r);
            if (PASS == 2) {
                const bool valid = col < ncol_g;
                const int qi = valid ? col / p.group : 0;
                const int h = g * p.group + (valid ? col % p.group : 0);
                norm[cb][r] = valid ? p.lse2[(int64_t)qi * p.hq + h] * p.lse_factor : INFINITY;
            } else {
                msc[cb][r] = 0.f;
                lsum[cb][r] = 0.f;
                tsum[cb][r] = 0.f;
            }
        }

    f32x16 s_a[NCB][2], s_b[NCB][2];   // S of one 64-key tile: [column block][key block]

    // ---- prologue --------------------------------------------------------------------------
#pragma unroll
    for (int T = 0; T < NS - 1; ++T) dma_tile(T);
    wait_vm<FILLS * (NS - 2)>();   // tile 0
    __syncthreads();
    {
        const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                          0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 16; ++i) {   // S(0), operands through the ring two at a time
            if ((i & 1) == 0) {
                load_op(0, 0, i, i & 7);
                load_op(0, 0, i + 1, (i + 1) & 7);
            }
            s_a[0][i & 1] = mfma32(qreg[0][i >> 1], kq[i & 7], i < 2 ? z : s_a[0][i & 1]);
        }
    }
    wait_vm<FILLS * (NS - 3)>();   // tile 1
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kLook; ++i) load_op(1, 1, i, i);
    wait_vm<FILLS * (NS - 4)>();   // tile 2 (the look-ahead of tile 0's last MFMAs reads it)
    __syncthreads();

    // exponents of the two keys of column (CB, R) of the tile in S
#define PKV_SCORE_PREP(S, CB, R, RAGGED)                                                 \
    {                                                                                    \
        float x0_ = S[CB][0][R], x1_ = S[CB][1][R];                                      \
        if (PASS == 1 && (RAGGED)) {                                                     \
            if (t0_ + l32 >= key_end) x0_ = -INFINITY;                                   \
            if (t0_ + 32 + l32 >= key_end) x1_ = -INFINITY;                              \
        }                                                                                \
        const float ref_ = PASS == 1 ? msc[CB][R] : norm[CB][R];                         \
        xa_ = x0_ * c2 - ref_;                                                           \
        xb_ = x1_ * c2 - ref_;                                                           \
    }
    // the pending pair of probabilities (pe0_, pe1_) belongs to column (CB, R)
#define PKV_SCORE_ADD(CB, R)                                                             \
    {                                                                                    \
        if (PASS == 1) {                                                                 \
            lsum[CB][R] += tsum[CB][R];   /* the previous tile's sum */                  \
            tsum[CB][R] = pe0_ + pe1_;                                                   \
            /* one instruction: fmaxf would first quiet a signalling NaN (a second  */   \
            /* v_max); a NaN sum needs no rescue and the hardware maximum drops it  */   \
            asm volatile("v_max_f32 %0, %0, %1" : "+v"(tmax_) : "v"(tsum[CB][R]));       \
            asm volatile("" : "+v"(lsum[CB][R]), "+v"(tsum[CB][R]));                     \
        } else {                                                                         \
            ksum[0] += pe0_;                                                             \
            ksum[1] += pe1_;                                                             \
            asm volatile("" : "+v"(ksum[0]), "+v"(ksum[1]));                             \
        }                                                                                \
    }

    // One tile: CUR = S(T) is turned into sums while NXT = S(T+1) is formed; the operand of
    // MFMA i + kLook (of tile T+1, or of tile T+2 behind the tile's end) is requested after
    // MFMA i.  ST1, ST2 = the ring stages of tiles T+1 and T+2 if known at compile time, else -1.
#define PKV_SCORE_TILE(CUR, NXT, T, ST1, ST2, RAGGED)                                            \
    {                                                                                    \
        const int t0_ = key_begin + (T) * kTile;                                         \
        dma_tile((T) + NS - 1);                                                          \
        float tmax_ = 0.f;   /* largest pair sum of the tile (pass 1) */                 \
        float xa_, xb_, pe0_ = 0.f, pe1_ = 0.f;                                          \
        PKV_SCORE_PREP(CUR, 0, 0, RAGGED)                                                \
        _Pragma("unroll") for (int kc = 0; kc < KC; ++kc) {                              \
            _Pragma("unroll") for (int q4 = 0; q4 < 2; ++q4) {                           \
                const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,               \
                                   0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};              \
                const int i_ = kc * 2 + q4;                                              \
                NXT[0][q4] = mfma32(qreg[0][kc], kq[i_ & 7], kc == 0 ? z_ : NXT[0][q4]); \
                if (i_ + kLook < 16) load_op((T) + 1, ST1, i_ + kLook, (i_ + kLook) & 7); \
                else load_op((T) + 2, ST2, i_ + kLook - 16, (i_ + kLook) & 7);           \
                /* softmax step: column (scb_, sr_), keys of both key blocks.  The    */ \
                /* exponents were formed one step earlier and the results are added   */ \
                /* one step later, so nothing waits on the transcendental unit.       */ \
                const int step_ = i_, scb_ = step_ >> 4, sr_ = step_ & 15;               \
                const float e0_ = __builtin_amdgcn_exp2f(xa_);                           \
                const float e1_ = __builtin_amdgcn_exp2f(xb_);                           \
                if (step_ < 16 * NCB - 1) {                                              \
                    const int ncb_ = (step_ + 1) >> 4, nr_ = (step_ + 1) & 15;           \
                    PKV_SCORE_PREP(CUR, ncb_, nr_, RAGGED)                               \
                }                                                                        \
                if (step_ > 0) {                                                         \
                    const int pcb_ = (step_ - 1) >> 4, pr_ = (step_ - 1) & 15;           \
                    PKV_SCORE_ADD(pcb_, pr_)                                             \
                }                                                                        \
                pe0_ = e0_;                                                              \
                pe1_ = e1_;                                                              \
                (void)scb_; (void)sr_;                                                   \
                asm volatile("" : "+v"(pe0_), "+v"(pe1_), "+v"(xa_), "+v"(xb_));         \
                __builtin_amdgcn_sched_barrier(0);                                       \
            }                                                                            \
        }                                                                                \
        PKV_SCORE_ADD(NCB - 1, 15)                                                       \
        if (PASS == 1) {                                                                 \
            /* an infinite sum shows here too; a NaN does not, and needs no rescue */  \
            if (__builtin_expect(__any(!(tmax_ < kGrow)), 0)) {                          \
                /* some sum left the safe range: raise the references to this tile's  */ \
                /* maxima where they are larger, rescale, form the tile's sums again  */ \
                _Pragma("unroll") for (int cb = 0; cb < NCB; ++cb)                       \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) {                         \
                    float x0_ = CUR[cb][0][r], x1_ = CUR[cb][1][r];                      \
                    if (t0_ + l32 >= key_end) x0_ = -INFINITY;                           \
                    if (t0_ + 32 + l32 >= key_end) x1_ = -INFINITY;                      \
                    const float mx_ = fmaxf(x0_, x1_) * c2;                              \
                    if (mx_ > msc[cb][r] || !(lsum[cb][r] > 0.f)) {                      \
                        /* (a lane that has seen no key yet takes the tile's maximum) */ \
                        const float ms_ = mx_ == -INFINITY ? 0.f : mx_;                  \
                        lsum[cb][r] *= __builtin_amdgcn_exp2f(msc[cb][r] - ms_);         \
                        msc[cb][r] = ms_;                                                \
                    }                                                                    \
                    tsum[cb][r] = __builtin_amdgcn_exp2f(x0_ * c2 - msc[cb][r]) +        \
                                  __builtin_amdgcn_exp2f(x1_ * c2 - msc[cb][r]);         \
                }                                                                        \
            }                                                                            \
        } else {                                                                         \
            /* the other half of the wave holds the other 16 columns of each block */    \
            float tot_[2];                                                               \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) {                           \
                const auto sw_ = __builtin_amdgcn_permlane32_swap(                       \
                    __float_as_uint(ksum[kb]), __float_as_uint(ksum[kb]), false, false); \
                tot_[kb] = __uint_as_float(sw_[0]) + __uint_as_float(sw_[1]);            \
                ksum[kb] = 0.f;                                                          \
            }                                                                            \
            float* const part_ =                                                         \
                p.part_score + ((int64_t)(g * p.n_cblk + cblk) * 4 + (wave & 3)) * p.n_ctx; \
            if (NW == 4) {                                                               \
                _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) {                       \
                    const int key_ = t0_ + kb * 32 + l32;                                \
                    if (hh == 0 && key_ < key_end) part_[key_] = tot_[kb];               \
                }                                                                        \
            } else if (wave >= 4) {                                                      \
                /* read by wave - 4 after this tile's barrier, written again two tiles on */ \
                if (hh == 0) {                                                           \
                    s_pair[(T) & 1][wave - 4][l32] = tot_[0];                            \
                    s_pair[(T) & 1][wave - 4][32 + l32] = tot_[1];                       \
                }                                                                        \
            } else {                                                                     \
                /* the previous tile: the partner's sums are in LDS since its barrier */ \
                if (pend_t0 >= 0) {                                                      \
                    _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) {                   \
                        const int key_ = pend_t0 + kb * 32 + l32;                        \
                        if (hh == 0 && key_ < key_end)                                   \
                            part_[key_] = pend[kb] + s_pair[((T) - 1) & 1][wave][kb * 32 + l32]; \
                    }                                                                    \
                }                                                                        \
                pend[0] = tot_[0];                                                       \
                pend[1] = tot_[1];                                                       \
                pend_t0 = t0_;                                                           \
            }                                                                            \
        }                                                                                \
        wait_vm<2 * FILLS>();   /* tile T+3 has landed (loads and the stores above complete */ \
        __syncthreads(); /* in order among themselves; this leaves room for the two youngest) */ \
    }

    // the reference of pass 1 starts as the maximum over the first tile (per lane)
    if (PASS == 1) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float x0 = s_a[cb][0][r], x1 = s_a[cb][1][r];
                if (key_begin + l32 >= key_end) x0 = -INFINITY;
                if (key_begin + 32 + l32 >= key_end) x1 = -INFINITY;
                const float mx = fmaxf(x0, x1);
                msc[cb][r] = mx == -INFINITY ? 0.f : mx * c2;
            }
    }

    // only the last tile of a split can reach past key_end
    const bool last_ragged = key_begin + n_iter * kTile > key_end;
    int T = 0;
    // once round the ring per trip: T is a multiple of NS = 6 here, so every stage is a constant
    for (; T + 6 < n_iter; T += 6) {
        PKV_SCORE_TILE(s_a, s_b, T, 1, 2, false)
        PKV_SCORE_TILE(s_b, s_a, T + 1, 2, 3, false)
        PKV_SCORE_TILE(s_a, s_b, T + 2, 3, 4, false)
        PKV_SCORE_TILE(s_b, s_a, T + 3, 4, 5, false)
        PKV_SCORE_TILE(s_a, s_b, T + 4, 5, 0, false)
        PKV_SCORE_TILE(s_b, s_a, T + 5, 0, 1, false)
    }
    for (; T + 2 < n_iter; T += 2) {
        PKV_SCORE_TILE(s_a, s_b, T, -1, -1, false)
        PKV_SCORE_TILE(s_b, s_a, T + 1, -1, -1, false)
    }
    if (T + 2 == n_iter) {
        PKV_SCORE_TILE(s_a, s_b, T, -1, -1, false)
        if (last_ragged) PKV_SCORE_TILE(s_b, s_a, T + 1, -1, -1, true)
        else PKV_SCORE_TILE(s_b, s_a, T + 1, -1, -1, false)
    } else {
        if (last_ragged) PKV_SCORE_TILE(s_a, s_b, T, -1, -1, true)
        else PKV_SCORE_TILE(s_a, s_b, T, -1, -1, false)
    }
    wait_vm<0>();   // nothing may still be writing LDS when the workgroup retires
    if (PASS == 2 && NW == 8 && wave < 4 && pend_t0 >= 0) {
        // the last tile's sums (its barrier has passed: the partner's are in LDS)
        float* const part = p.part_score + ((int64_t)(g * p.n_cblk + cblk) * 4 + wave) * p.n_ctx;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const int key = pend_t0 + kb * 32 + l32;
            if (hh == 0 && key < key_end)
                part[key] = pend[kb] + s_pair[(n_iter - 1) & 1][wave][kb * 32 + l32];
        }
    }
#undef PKV_SCORE_TILE
#undef PKV_SCORE_PREP
#undef PKV_SCORE_ADD

    // ---- pass 1 epilogue: the 32 key lanes of a column meet through LDS -----------------------
    if (PASS == 1) {
        __syncthreads();   // the ring is idle (all loads landed, all reads done)
        // [key lane j][column c] as float2 (reference * c2, sum); the column index is
        // rotated by j so that both the writes (32 lanes, one column) and the reads (64
        // consecutive columns, one j) spread over all banks
        float2* ex = reinterpret_cast<float2*>(smem);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = wave * (32 * NCB) + cb * 32 + 8 * (r / 4) + 4 * hh + (r % 4);
                ex[l32 * 256 + ((c + l32) & 255)] =
                    make_float2(msc[cb][r], lsum[cb][r] + tsum[cb][r]);
            }
        __syncthreads();
        if (tid >= 256) return;   // one thread per column from here on
        const int c = tid;
        float m = -INFINITY, l = 0.f;   // running (reference * c2, sum) over the lanes with keys
        for (int j = 0; j < 32; ++j) {
            const float2 v = ex[j * 256 + ((c + j) & 255)];
            if (!(v.y > 0.f)) continue;   // that lane saw no key of the split
            const float mn = fmaxf(m, v.x);
            l = l * __builtin_amdgcn_exp2f(m - mn) + v.y * __builtin_amdgcn_exp2f(v.x - mn);
            m = mn;
        }
        const int col = cblk * 256 + c;
        if (col < ncol_g) {
            const int qi = col / p.group;
            const int h = g * p.group + col % p.group;
            float* dst = p.part_ml + ((int64_t)split * p.nq * p.hq + (int64_t)qi * p.hq + h) * 2;
            dst[0] = m == -INFINITY ? -INFINITY : m / c2;   // back to raw logits
            dst[1] = l;
        }
    }
}

}  // namespace

ScorePlan plan_score_dma128(const pkv_layer_cfg& cfg, int64_t n_ctx, int64_t nq) {
    const int group = cfg.n_q_heads / cfg.n_kv_heads;
    ScorePlan sp;
    sp.n_cblk = (int)ceil_div(nq * group, 256);
    // as many key splits as keep the launch within one round of a 256-CU part (a 257th
    // workgroup would double the time of the launch)
    int64_t want = 256 / ((int64_t)sp.n_cblk * cfg.n_kv_heads);
    const int64_t max_splits = ceil_div(n_ctx, 4 * kTile);
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    const int64_t len = ceil_div(ceil_div(n_ctx, want), kTile) * kTile;
    sp.split_len = (int)len;
    sp.n_splits = (int)ceil_div(n_ctx, len);
    sp.n_parts = sp.n_cblk * cfg.n_kv_heads * 4;
    return sp;
}

bool score_dma128_supported(const pkv_layer_cfg& cfg, int64_t n_ctx, int64_t nq) {
    const int group = cfg.n_kv_heads > 0 ? cfg.n_q_heads / cfg.n_kv_heads : 0;
    // 32-bit byte offsets inside one split of K; int indices elsewhere
    return cfg.dtype == PKV_BF16 && cfg.head_dim == D && group >= 1 && nq > 0 && n_ctx > 0 &&
           n_ctx < (1 << 30) && nq * cfg.n_q_heads < (1 << 30) &&
           (int64_t)(kTile + 1) * cfg.n_kv_heads * D * 2 < (int64_t)1 << 31;
}

pkv_status launch_score_dma128(int pass, const ScoreParams& p, hipStream_t st) {
    static std::atomic<bool> configured{false};   // set twice at worst: the calls are idempotent
    if (!configured.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(score_dma128_kernel<1, kScoreWaves>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(score_dma128_kernel<2, kScoreWaves>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess)
            return PKV_ERR_LAUNCH;
        configured.store(true, std::memory_order_release);
    }
    if (!p.q || !p.k || (pass == 1 ? !p.part_ml : (!p.lse2 || !p.part_score)))
        return PKV_ERR_NULL;
    const int64_t grid = (int64_t)p.n_cblk * p.n_splits * p.hkv;
    if (pass == 1)
        hipLaunchKernelGGL((score_dma128_kernel<1, kScoreWaves>), dim3((unsigned)grid),
                           dim3(64 * kScoreWaves), kLdsBytes, st, p);
    else
        hipLaunchKernelGGL((score_dma128_kernel<2, kScoreWaves>), dim3((unsigned)grid),
                           dim3(64 * kScoreWaves), kLdsBytes, st, p);
    return launch_status();
}

}  // namespace pkv
