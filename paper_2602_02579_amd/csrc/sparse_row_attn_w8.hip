// Step 5, head_dim 128, bf16, eight waves per workgroup.
// (Paper: Sec. 4.3 Stage II - complete recomputation, but only for the selected
// tokens; Sec. 5.3 - this attention over the long cache dominates the cost.)
//
// Same tile, same LDS layout, same arithmetic as attn_dma128_kernel
// (sparse_row_attn_dma.hip):
//     S^T = K Q^T,   O^T += V^T P^T     (v_mfma_f32_32x32x16_bf16)
// with a fixed softmax reference per column and marked tiles redone by the exact
// kernel.  What differs is who does the work.  There a workgroup is 4 waves of 64
// columns, one wave per SIMD, and the softmax arithmetic of a wave can only hide
// under its own MFMAs: the counters show the matrix pipe busy 63 % of the time, the
// rest is VALU work and waits of the one instruction stream.  Here a workgroup is 8
// waves of 32 columns, two waves per SIMD (~250 registers each): while one wave
// issues softmax arithmetic or waits for LDS, the other wave's MFMAs run.  The price
// is LDS traffic - every wave reads the whole K and V^T tile for half the MFMAs, 1 KB
// per MFMA instead of 512 B - which the 64-bank LDS of this part carries.
//
// A wave's sub-step (32 keys) is 16 MFMAs in a three-deep software pipeline:
//     S^T(u+2) from K operands loaded one sub-step earlier,
//     P(u+1)   from S^T(u+1), one score after each MFMA,
//     O^T     += V^T(u) P^T(u).
// Every result is consumed a full sub-step after it was produced.
//
// Two instantiations: <false> reads V^T tiles from a transposed copy of the value cache
// that a pre-pass makes; <true> fills LDS with the value rows as the cache holds them and
// transposes them on the way out (ds_read_b64_tr_b16: 1.5 instead of 1 LDS instruction per
// MFMA, a loop ~2.5 % slower, no pre-pass).  The launcher picks by problem size.
#include <algorithm>
#include <atomic>

#include "attn_common.h"

namespace pkv {

namespace {

constexpr int D = 128;
constexpr int KC = D / 16;             // contraction chunks of S^T
constexpr int DB = D / 32;             // 32-row blocks of O^T
constexpr int NS = 4;                  // LDS stages per operand
constexpr int NW = 8;                  // waves per workgroup
constexpr int kThreads = NW * 64;
constexpr int kStageK = kBN * D * 2;   // bytes: 64 keys x 256 B
constexpr int kStageV = D * kBN * 2;   // bytes: 128 d-rows x 128 B
constexpr int kLdsBytes = NS * (kStageK + kStageV);
constexpr int kStealLag = 2;   // tiles another kv head must be behind before a workgroup helps it

// 16 bytes per lane from global memory straight into LDS: lane i of the wave
// writes LDS bytes [lds_base + 16 i, +16); lds_base must be wave-uniform.
__device__ __forceinline__ void dma16(const void* gbase, uint32_t voffset, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2"
        :
        : "s"(lds_base), "v"(voffset), "s"(gbase)
        : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// O^T accumulators pinned to the accumulation registers (never touched by the VALU
// inside the loop)
__device__ __forceinline__ void mfma32_acc(bf16x8 a, bf16x8 b, f32x16& c) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}

// Four 16-bit elements per lane through the transposing LDS read: within each group of 16
// lanes, lane i receives as element e the element i % 4 of what lane 4 e + i / 4 addressed.
// With lane 4 e + j addressing V[key + e][d0 + 4 j .. d0 + 4 j + 3] of a tile stored key-major,
// lane i ends up with V[key .. key + 3][d0 + i]: an A-operand fragment of V^T.
typedef short i16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char* ptr) {
    const i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) i16x4*)ptr);
    return __builtin_bit_cast(bf16x4, v);
}

// kNatV: the values are read from the cache as it is (key-major) and transposed on their
// way out of LDS; otherwise from a V^T copy made by a pre-pass.
template <bool kNatV>
__global__ __launch_bounds__(kThreads) void attn_w8_kernel(AttnParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_red[NW];
    __shared__ int s_job;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5;
    const int l32 = lane & 31;

    // Work distribution: one workgroup per CU claims (kv head, row tile[, key range]) jobs,
    // heaviest first, from one counter per kv head; it prefers its home head (whose K/V its
    // XCD's L2 holds) unless another head is kStealLag or more jobs behind.
    const int home = blockIdx.x % p.hkv;
    const int jobs_per_head = p.n_tiles * p.dma_splits;
  for (;;) {
    if (tid == 0) {
        int job = -1;
        // at most hkv failed claims: each one finds a head exhausted for good
        for (int attempt = 0; attempt <= p.hkv && job < 0; ++attempt) {
            int best = home;
            int best_c = __hip_atomic_load(&p.queue[home], __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
            if (best_c < jobs_per_head) best_c -= kStealLag;
            for (int q = 1; q < p.hkv; ++q) {
                int y = home + q;
                if (y >= p.hkv) y -= p.hkv;
                const int c = __hip_atomic_load(&p.queue[y], __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
                if (c < best_c) {
                    best_c = c;
                    best = y;
                }
            }
            if (best_c >= jobs_per_head) break;   // nothing left anywhere
            const int j = atomicAdd(&p.queue[best], 1);
            if (j < jobs_per_head) job = best * jobs_per_head + j;
        }
        s_job = job;
    }
    __syncthreads();
    const int job = __builtin_amdgcn_readfirstlane(s_job);
    if (job < 0) break;   // block-uniform: every head is exhausted
    const int g = job / jobs_per_head;
    const int within = job - g * jobs_per_head;
    const int tile = p.n_tiles - 1 - within / p.dma_splits;
    const int split = within % p.dma_splits;
    const int kb = split * p.dma_split_len;                      // a multiple of kBN
    const int n_keys_job = min(p.n_keys - kb, p.dma_split_len);  // keys the job may touch

    // ---- this lane's column ---------------------------------------------------------------
    const int col = wave * 32 + l32;
    const int rl = col / p.group;
    const int row = tile * p.bm + rl;
    const int head = g * p.group + col % p.group;
    const bool valid = rl < p.bm && row < p.m;
    // last key of this job's range that the column sees (negative: none).  Clamped to the
    // range: the pipeline forms the probabilities of one sub-step beyond the last tile and
    // adds them to the sum, so whatever lies behind the range has to be masked like the keys
    // behind the row's own position.
    const int limit = valid ? min(p.row_pos[row] - kb, n_keys_job - 1) : -1;
    int lmax = limit, lmin = valid ? limit : 0x7fffffff;
    for (int o = 32; o > 0; o >>= 1) {
        lmax = max(lmax, __shfl_xor(lmax, o, 64));
        lmin = min(lmin, __shfl_xor(lmin, o, 64));
    }
    if (lane == 0) s_red[wave] = lmax;
    __syncthreads();
    int tile_max = -1;
#pragma unroll
    for (int w = 0; w < NW; ++w) tile_max = max(tile_max, s_red[w]);
    const int key_end = min(tile_max + 1, n_keys_job);
    const int n_iter = __builtin_amdgcn_readfirstlane((key_end + kBN - 1) / kBN);
    if (n_iter <= 0) {        // block-uniform: no valid row, or no row reaches this range
        if (tid == 0 && p.dma_splits == 1) p.flags[tile * p.hkv + g] = 0;
        continue;
    }
    // sub-steps [0, u_unm) lie entirely at or below every limit of this wave; a wave without
    // a valid column has nothing to mask
    const int u_unm = __builtin_amdgcn_readfirstlane(lmin == 0x7fffffff ? 0x3fffffff
                                                                        : (lmin + 1) / 32);

    // ---- Q as B operands ---------------------------------------------------------------------
    bf16x8 qreg[KC];
    {
        const bf16_t* qp = p.q + ((int64_t)row * p.hq + head) * D + hh * 8;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            if (valid) {
                qreg[kc] = *reinterpret_cast<const bf16x8*>(qp + kc * 16);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) qreg[kc][e] = (bf16_t)0.0f;
            }
        }
    }

    float m_run = -INFINITY, l_run = 0.f;
    f32x16 o_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;

    // ---- global -> LDS ------------------------------------------------------------------------
    // K stage: key row r at byte r*256, 16-byte chunk c at c ^ (r & 15).  V^T stage: row d at
    // byte d*128, chunk c at c ^ ((d >> 1) & 7).  A wave instruction fills 1 KB; wave w owns K
    // rows [8w, 8w+8) and V^T rows [16w, 16w+16) of every tile: two instructions each.
    // Key-major V stage (kNatV): key row r at byte r*256, chunk c at c ^ (4 (r & 3)), so that
    // the four rows x 64 bytes a half wave reads in one transposing instruction cover all 64
    // banks once; wave w owns rows [8w, 8w+8).
    const uint32_t lds_k = (uint32_t)(uintptr_t)smem;
    const uint32_t lds_v = lds_k + NS * kStageK;
    const uint32_t k_row_bytes = (uint32_t)p.hkv * D * 2;
    uint32_t voff_k[2], voff_v[2], kofs_last[2], vofs_last[2];
    {
        const int last = (n_keys_job - 1) % kBN;   // last row of the (possibly ragged) last tile
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = 8 * wave + 4 * i + (lane >> 4);
            const uint32_t chunk = (uint32_t)(((lane & 15) ^ (r & 15)) * 16);
            voff_k[i] = (uint32_t)r * k_row_bytes + chunk;
            kofs_last[i] = (uint32_t)min(r, last) * k_row_bytes + chunk;
            if (kNatV) {
                const uint32_t vchunk = (uint32_t)(((lane & 15) ^ (4 * (r & 3))) * 16);
                voff_v[i] = (uint32_t)r * k_row_bytes + vchunk;
                vofs_last[i] = (uint32_t)min(r, last) * k_row_bytes + vchunk;
            } else {
                const int d = 16 * wave + 8 * i + (lane >> 3);
                voff_v[i] =
                    (uint32_t)d * (uint32_t)p.n_pad * 2u + (((lane & 7) ^ ((d >> 1) & 7)) * 16);
                vofs_last[i] = voff_v[i];
            }
        }
    }
    const uint32_t lds_k_wave = __builtin_amdgcn_readfirstlane(lds_k + wave * 8 * 256);
    const uint32_t lds_v_wave = __builtin_amdgcn_readfirstlane(lds_v + wave * 16 * 128);
    const bf16_t* const k_head = p.k + ((int64_t)kb * p.hkv + g) * D;
    const bf16_t* const v_head = kNatV ? p.v + ((int64_t)kb * p.hkv + g) * D
                                       : p.vt + (int64_t)g * D * p.n_pad + kb;

    // K tile T / V^T tile T (clamped to the last tile) into their ring slots, both instructions
#define W8_DMA_K(T)                                                                      \
    {                                                                                    \
        const int t_ = min((T), n_iter - 1);                                             \
        const bf16_t* gb_ = k_head + (int64_t)t_ * kBN * p.hkv * D;                      \
        const bool full_ = t_ * kBN + kBN <= n_keys_job;                                 \
        _Pragma("unroll") for (int i = 0; i < 2; ++i)                                    \
            dma16(gb_, full_ ? voff_k[i] : kofs_last[i],                                 \
                  lds_k_wave + ((T) & 3) * kStageK + i * 1024);                          \
    }
#define W8_DMA_V(T)                                                                      \
    {                                                                                    \
        const int t_ = min((T), n_iter - 1);                                             \
        const bf16_t* gb_ = kNatV ? v_head + (int64_t)t_ * kBN * p.hkv * D               \
                                  : v_head + t_ * kBN;                                   \
        const bool full_ = t_ * kBN + kBN <= n_keys_job;                                 \
        _Pragma("unroll") for (int i = 0; i < 2; ++i)                                    \
            dma16(gb_, full_ ? voff_v[i] : vofs_last[i],                                 \
                  lds_v_wave + ((T) & 3) * kStageV + i * 1024);                          \
    }
    // the four fill instructions of a tile body (K tile J+4, V^T tile J+2), one pair per
    // sub-step, prepared once per tile
    const bf16_t* gbk_;
    const bf16_t* gbv_;
    bool k_full_, v_full_;
#define W8_DMA_PREP(J)                                                                   \
    {                                                                                    \
        const int tk_ = min((J) + 4, n_iter - 1);                                        \
        gbk_ = k_head + (int64_t)tk_ * kBN * p.hkv * D;                                  \
        k_full_ = tk_ * kBN + kBN <= n_keys_job;   /* wave-uniform */                    \
        const int tv_ = min((J) + 2, n_iter - 1);                                        \
        gbv_ = kNatV ? v_head + (int64_t)tv_ * kBN * p.hkv * D : v_head + tv_ * kBN;     \
        v_full_ = tv_ * kBN + kBN <= n_keys_job;                                         \
    }
#define W8_DMA_ONE_K(I, SDK)                                                             \
    dma16(gbk_, k_full_ ? voff_k[I] : kofs_last[I], lds_k_wave + (SDK) * kStageK + (I) * 1024);
#define W8_DMA_ONE_V(I, SDV)                                                             \
    dma16(gbv_, v_full_ ? voff_v[I] : vofs_last[I], lds_v_wave + (SDV) * kStageV + (I) * 1024);

    // ---- LDS -> register operand addresses (bytes inside a stage) -----------------------------
    // A-row i of a 32-key block reads key swap_bits23(i) of that block, so that accumulator
    // register r of lane half hh holds key 16*(r/8) + 8*hh + r%8.
    const int prow = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    uint32_t kaddr[KC], vaddr[4];
    {
        const uint32_t a0 = prow * 256 + (((prow & 15) ^ hh) * 16);
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) kaddr[kc] = a0 ^ (kc << 5);
        if (kNatV) {
            // vaddr[db]: the 8 bytes this lane addresses for the d-block db of a 16-key chunk
            // (row 8 hh + e of the chunk, d = 32 db + 16 gh + 4 j .. + 3)
            const int e = (lane >> 2) & 3, j = lane & 3, gh = (lane >> 4) & 1;
#pragma unroll
            for (int db = 0; db < 4; ++db)
                vaddr[db] = (uint32_t)((8 * hh + e) * 256 +
                                       (((db ^ e) * 4 + gh * 2 + (j >> 1)) * 16) + (j & 1) * 8);
        } else {
            const uint32_t v0 = l32 * 128 + ((((l32 >> 1) & 7) ^ hh) * 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) vaddr[q] = v0 ^ (q << 5);
        }
        // the value stages lie behind the 64 KB of key stages: with that base inside the lane's
        // address every stage and block offset of a value read fits the 16-bit immediate of
        // the LDS instruction, and no address arithmetic is left in the loop
#pragma unroll
        for (int q = 0; q < 4; ++q) vaddr[q] += NS * kStageK;
    }
    const float c2 = p.scale_log2;

    f32x16 s_a, s_b;          // S^T of even / odd sub-steps
    bf16x8 pb_a[2], pb_b[2];  // P^T of even / odd sub-steps: [16-key half]
    bf16x8 ka[KC], va[2][DB];
    float rs = 0.f;           // this lane's sum of the probabilities being produced
    float msc;                // reference maximum times c2 (0 while it is -inf)
    constexpr float kGrow = 1.0e24f;   // ~2^80
    float rs_max = 0.f;
    float e_half = 0.f;
    float x_next;

#define W8_LOAD_KA(ST, H)                                                                \
    _Pragma("unroll") for (int kc = 0; kc < KC; ++kc)                                    \
        ka[kc] = *reinterpret_cast<const bf16x8*>(                                       \
            smem + (ST) * kStageK + (H) * 32 * 256 + kaddr[kc]);
    // one operand at a time: element KCI of the K half (ST, H); element (KK, DBI) of the V^T
    // half (ST, H)
#define W8_LOAD_KA1(ST, H, KCI)                                                          \
    ka[KCI] = *reinterpret_cast<const bf16x8*>(                                          \
        smem + (ST) * kStageK + (H) * 32 * 256 + kaddr[KCI]);
#define W8_LOAD_VA1(ST, H, KK, DBI)                                                      \
    if (kNatV) {                                                                         \
        const unsigned char* a_ = smem + (ST) * kStageV +                                \
                                  (32 * (H) + 16 * (KK)) * 256 + vaddr[DBI];             \
        const bf16x4 lo_ = lds_read_tr(a_), hi_ = lds_read_tr(a_ + 4 * 256);             \
        va[KK][DBI] = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);         \
    } else {                                                                             \
        va[KK][DBI] = *reinterpret_cast<const bf16x8*>(                                  \
            smem + (ST) * kStageV + (DBI) * 32 * 128 + vaddr[2 * (H) + (KK)]);           \
    }

    // exponent of element R of score buffer S whose first key is T0
#define W8_SM_PREP(S, R, T0, MASK)                                                       \
    {                                                                                    \
        float x_ = S[R];                                                                 \
        if (MASK) {                                                                      \
            const int key_ = (T0) + 16 * ((R) / 8) + 8 * hh + (R) % 8;                   \
            if (key_ > limit) x_ = -INFINITY;                                            \
        }                                                                                \
        x_next = x_ * c2 - msc;                                                          \
    }
    // probability of element R (exponent prepared one step earlier) into PB; prepares the
    // exponent of element RN of SN (first key T0N) in between
#define W8_SM_STEP(PB, R, SN, RN, T0N, MASK)                                             \
    {                                                                                    \
        const float e_ = __builtin_amdgcn_exp2f(x_next);                                 \
        W8_SM_PREP(SN, RN, T0N, MASK)                                                    \
        rs += e_;                                                                        \
        if ((R) % 2 == 0) {                                                              \
            e_half = e_;                                                                 \
            asm volatile("" : "+v"(rs), "+v"(e_half), "+v"(x_next));                     \
        } else {                                                                         \
            PB[(R) / 8][(R) % 8 - 1] = (bf16_t)e_half;                                   \
            PB[(R) / 8][(R) % 8] = (bf16_t)e_;                                           \
            asm volatile("" : "+v"(rs), "+v"(PB[(R) / 8]), "+v"(x_next));                \
        }                                                                                \
    }

    // One 32-key sub-step u.  SCUR = S^T(u+1) (complete), SNXT receives S^T(u+2) from the
    // operands in ka; PCUR = P(u) (complete), PNXT receives P(u+1); (KST, KH) name the K
    // half tile of sub-step u+3, (VST, VH) the V^T half tile of sub-step u; T0N is the first
    // key of sub-step u+1.  I = which of the tile's two fill pairs goes out here.
#define W8_SUBSTEP(SCUR, SNXT, PCUR, PNXT, KST, KH, VST, VH, T0N, MASK, I, SDK, SDV)     \
    {                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                               \
        W8_DMA_ONE_K(I, SDK)                                                             \
        __builtin_amdgcn_sched_barrier(0);                                               \
        /* every MFMA frees one operand; the operand that the other group needs eight   \
           MFMAs later is requested into its place, so K and V^T operands together      \
           never hold more than nine registers' worth of tiles */                       \
        _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_) {                               \
            const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,                   \
                               0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};                  \
            SNXT = mfma32(ka[i_], qreg[i_], i_ == 0 ? z_ : SNXT);                        \
            W8_LOAD_VA1(VST, VH, i_ >> 2, i_ & 3)                                        \
            W8_SM_STEP(PNXT, i_, SCUR, i_ + 1, T0N, MASK)                                \
            __builtin_amdgcn_sched_barrier(0);                                           \
        }                                                                                \
        W8_DMA_ONE_V(I, SDV)                                                             \
        __builtin_amdgcn_sched_barrier(0);                                               \
        _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_) {                               \
            const int kk_ = i_ >> 2, db_ = i_ & 3;                                       \
            mfma32_acc(va[kk_][db_], PCUR[kk_], o_acc[db_]);                             \
            W8_LOAD_KA1(KST, KH, i_)                                                     \
            if (i_ < 7) { W8_SM_STEP(PNXT, 8 + i_, SCUR, 9 + i_, T0N, MASK) }            \
            else { W8_SM_STEP(PNXT, 15, SNXT, 0, (T0N) + 32, MASK) }                     \
            __builtin_amdgcn_sched_barrier(0);                                           \
        }                                                                                \
        l_run += rs;                                                                     \
        rs_max = fmaxf(rs_max, rs);                                                      \
        rs = 0.f;                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                               \
    }

    // one 64-key tile J: sub-steps 2J, 2J+1.  K halves read: tile J+1 half 1 (stage SK1) and
    // tile J+2 half 0 (stage SK2); V^T tile J in stage SV0; K(J+4) -> stage SV0's index (the
    // slot of K(J)), V^T(J+2) -> stage SK2's index.
#define W8_TILE(J, SK1, SK2, SV0, MASK)                                                  \
    {                                                                                    \
        const int t0_tile_ = (J) * kBN;                                                  \
        W8_DMA_PREP(J)                                                                   \
        W8_SUBSTEP(s_b, s_a, pb_a, pb_b, SK1, 1, SV0, 0, t0_tile_ + 32, MASK, 0, SV0, SK2) \
        W8_SUBSTEP(s_a, s_b, pb_b, pb_a, SK2, 0, SV0, 1, t0_tile_ + 64, MASK, 1, SV0, SK2) \
        wait_vm<4>();   /* K(J+3), V^T(J+1) have landed; the 4 newest loads stay in flight */ \
        __syncthreads();                                                                 \
    }

    // ---- prologue -------------------------------------------------------------------------
    W8_DMA_K(0)
    W8_DMA_V(0)
    W8_DMA_K(1)
    W8_DMA_K(2)
    wait_vm<0>();
    __syncthreads();
    W8_DMA_K(3)
    W8_DMA_V(1)
    W8_LOAD_KA(0, 0)
    {
        const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                           0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s_a = mfma32(ka[0], qreg[0], z_);
#pragma unroll
        for (int kc = 1; kc < KC; ++kc) s_a = mfma32(ka[kc], qreg[kc], s_a);
    }
    W8_LOAD_KA(0, 1)
    {
        const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                           0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s_b = mfma32(ka[0], qreg[0], z_);
#pragma unroll
        for (int kc = 1; kc < KC; ++kc) s_b = mfma32(ka[kc], qreg[kc], s_b);
    }
    W8_LOAD_KA(1, 0)            // operands of S^T(2)
    // the reference of the column: the maximum of its first 32 keys, fixed from here on
    {
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 16 * (r / 8) + 8 * hh + (r % 8);
            if (key <= limit) mx = fmaxf(mx, s_a[r]);
        }
        m_run = fmaxf(mx, __shfl_xor(mx, 32, 64));
        msc = (m_run == -INFINITY ? 0.f : m_run) * c2;
    }
    // P(0) in full
    W8_SM_PREP(s_a, 0, 0, true)
#pragma unroll
    for (int r = 0; r < 15; ++r) W8_SM_STEP(pb_a, r, s_a, r + 1, 0, true)
    W8_SM_STEP(pb_a, 15, s_b, 0, 32, true)
    l_run += rs;
    rs_max = fmaxf(rs_max, rs);
    rs = 0.f;
    // tile 0 already requests K(4) into the slot of K(0): every wave must be done reading it
    __syncthreads();

    // ---- main loop: four tiles per trip so that every LDS stage is a constant ----------------
    // tile j is mask free when every score it turns into a probability (sub-steps 2j+1, 2j+2
    // and the first element of 2j+3) lies at or below every limit of the wave: 2j + 3 < u_unm
    int n_unm = min(n_iter, max(0, (u_unm - 2) / 2));
    n_unm &= ~3;
    int j = 0;
    for (; j < n_unm; j += 4) {
        W8_TILE(j, 1, 2, 0, false)
        W8_TILE(j + 1, 2, 3, 1, false)
        W8_TILE(j + 2, 3, 0, 2, false)
        W8_TILE(j + 3, 0, 1, 3, false)
    }
    for (; j < n_iter; ++j) {
        W8_TILE(j, (j + 1) & 3, (j + 2) & 3, j & 3, true)
    }
    wait_vm<0>();   // nothing may still be writing LDS when the workgroup moves on
    // the last O^T MFMAs were issued behind the compiler's back: let them retire before the
    // accumulators are read
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

#undef W8_DMA_K
#undef W8_DMA_V
#undef W8_DMA_PREP
#undef W8_DMA_ONE_K
#undef W8_DMA_ONE_V
#undef W8_LOAD_KA
#undef W8_LOAD_KA1
#undef W8_LOAD_VA1
#undef W8_SM_PREP
#undef W8_SM_STEP
#undef W8_SUBSTEP
#undef W8_TILE

    // ---- epilogue ------------------------------------------------------------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    {
        const bool bad = !(rs_max < kGrow) || !(l_tot < 3.0e38f);
        const int wave_bad = __any(bad) ? 1 : 0;   // over all lanes, before the branch
        __syncthreads();                       // s_red held the tile limits so far
        if (lane == 0) s_red[wave] = wave_bad;
        __syncthreads();
        if (tid == 0) {
            int marked = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) marked |= s_red[w];
            int* const flag = &p.flags[tile * p.hkv + g];
            int* const count = &p.flags[p.n_tiles * p.hkv];   // behind the flags
            if (p.dma_splits == 1) {
                *flag = marked;
                if (marked) atomicAdd(count, 1);
            } else if (marked && atomicOr(flag, 1) == 0) {   // flags were cleared beforehand
                atomicAdd(count, 1);
            }
        }
    }
    if (valid) {
        const float inv = 1.f / l_tot;
        // A row whose keys all lie in the first range has its whole result in that range's
        // job: it is written as the final output there and never merged.  Every other row
        // leaves a normalised fp32 partial result per range it reaches.
        const int pos = min(p.row_pos[row], p.n_keys - 1);
        const bool direct = p.dma_splits == 1 || pos < p.dma_split_len;
        if (!direct) {
            if (pos >= kb) {   // else the row sees nothing of this range
                const int64_t colg = ((int64_t)split * p.m + row) * p.hq + head;
                float* op = p.part_o + colg * D + 4 * hh;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        f32x4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = o_acc[db][4 * r4 + e] * inv;
                        *reinterpret_cast<f32x4*>(op + db * 32 + r4 * 8) = v;
                    }
                if (hh == 0) p.part_lse[colg] = m_run * p.scale + logf(l_tot);
            }
        } else if (split == 0) {
            const int64_t colg = (int64_t)row * p.hq + head;
            bf16_t* op = p.out + colg * D + 4 * hh;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(o_acc[db][4 * r4 + e] * inv);
                    *reinterpret_cast<bf16x4*>(op + db * 32 + r4 * 8) = v;
                }
            if (hh == 0) {
                const float lse = m_run * p.scale + logf(l_tot);
                if (p.lse) p.lse[colg] = lse;
                // asked for only when every key the row sees is a context key: unsplit
                // launches whose keys are all context keys, and first-range rows (a range
                // boundary lies at the end of the context)
                if (p.lse_ctx) p.lse_ctx[colg] = lse;
            }
        }
    }
  }   // next job
}

}  // namespace

pkv_status launch_attn_w8_main(const AttnParams& p, int n_cu, hipStream_t st) {
    static std::atomic<bool> configured{false};   // set twice at worst: the calls are idempotent
    if (!configured.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(attn_w8_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(attn_w8_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess)
            return PKV_ERR_LAUNCH;
        configured.store(true, std::memory_order_release);
    }
    // one workgroup per CU (its LDS admits no second one), or per job if there are fewer
    const int64_t grid = std::min<int64_t>((int64_t)p.n_tiles * p.dma_splits * p.hkv, n_cu);
    if (p.v)   // the values as the cache holds them; p.vt is then not used
        hipLaunchKernelGGL(attn_w8_kernel<true>, dim3((unsigned)grid), dim3(kThreads), kLdsBytes,
                           st, p);
    else
        hipLaunchKernelGGL(attn_w8_kernel<false>, dim3((unsigned)grid), dim3(kThreads),
                           kLdsBytes, st, p);
    return launch_status();
}

}  // namespace pkv
