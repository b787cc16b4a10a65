// Step 5, head_dim 128, bf16: the attention kernel that the benchmark times.
// (Paper: Sec. 4.3 Stage II - complete recomputation, but only for the selected
// tokens; Sec. 5.3 - this attention over the long cache dominates the cost.)
//
// Tiling and register layouts are those of attn_mfma_kernel (see
// sparse_row_attn.hip): a workgroup of 4 waves owns 256 (row, head) columns of
// one kv head, everything is computed transposed,
//     S^T = K Q^T,   O^T += V^T P^T     (v_mfma_f32_32x32x16_bf16)
// and the probabilities go from the S^T accumulators straight into the second
// MFMA.  What is different here is how the kernel is kept busy:
//
// * One wave per SIMD (~450 registers), so MFMA and softmax work overlap only
//   inside one instruction stream.  On this chip a SIMD issues one VALU-class
//   instruction per 4 cycles and an MFMA 32x32x16 holds the matrix pipe for 8
//   such slots, so at most ~7 other instructions per MFMA are free.  The keys
//   of a 64-key tile are processed as two 32-key sub-steps of 32 MFMAs; the
//   softmax of a sub-step is cut into 16 pairs of scores and one pair follows
//   every second MFMA (see PKV_SUBSTEP), pinned with sched_barrier.
// * LDS -> register operand loads are issued one phase ahead of their MFMAs.
// * K and V^T tiles reach LDS by direct global->LDS loads (no staging
//   registers, no ds_write), 4 stages deep, issued three tiles ahead; the only
//   synchronisation per 64 keys is one s_waitcnt vmcnt + one barrier.  The
//   LDS tiles are unpadded; a 16-byte-chunk XOR swizzle (applied on the global
//   address side of the load) keeps the MFMA operand reads conflict free.
//   The loads are inline asm because the compiler would otherwise make every
//   LDS read wait for all outstanding global->LDS loads.
// * The reference maximum of a column is fixed after its first 32 keys (see
//   PKV_ACC): no maximum, no rescaling and no branch in the hot loop; tiles whose
//   probabilities leave the safe range are marked and redone by the exact kernel.
#include <algorithm>
#include <atomic>
#include <cstdlib>

#include "attn_common.h"

namespace pkv {

namespace {

constexpr int D = 128;
constexpr int KC = D / 16;             // contraction chunks of S^T
constexpr int DB = D / 32;             // 32-row blocks of O^T
constexpr int NS = 4;                  // LDS stages per operand
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

// O^T += V^T P^T with the accumulator tile pinned to the accumulation registers: the
// output accumulators are never touched by the VALU inside the loop, so they do not
// compete with the score tiles (which the softmax reads) for the ordinary registers.
// The compiler does not see through the statement: every operand it reads was written
// several instructions earlier, and the same accumulator recurs only every eighth MFMA.
__device__ __forceinline__ void mfma32_acc(bf16x8 a, bf16x8 b, f32x16& c) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

__global__ __launch_bounds__(kAttnThreads) void attn_dma128_kernel(AttnParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_red[kAttnThreads / 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int hh = lane >> 5;
    const int l32 = lane & 31;

    // Work distribution.  The launch is one workgroup per CU and every workgroup claims
    // (kv head, row tile) pairs until none are left: a row tile costs about one unit per
    // 64 keys below its largest limit, so with rows in position order the costs rise
    // linearly, there are only a few tiles per CU, and the CUs (and the XCDs, which do not
    // all run at the same speed) finish far apart when the hardware hands out whole
    // workgroups; claiming the next tile also costs much less than starting a workgroup.
    // Each kv head has a counter; tiles are claimed heaviest first.  Workgroup b starts
    // with head b mod hkv - with 8 kv heads that head's K/V stream is then shared through
    // the L2 of the XCD the workgroup runs on - and moves on to the following heads once
    // its own has nothing left.
    __shared__ int s_job;
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
            if (best_c < jobs_per_head) best_c -= kStealLag;   // prefer the own head
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
    // With few row tiles the keys of a tile are cut into dma_splits ranges, one job each
    // (normalised partial outputs, merged afterwards).  Everything below works in key
    // positions relative to the start of the job's range.
    const int split = within % p.dma_splits;
    const int kb = split * p.dma_split_len;                      // a multiple of kBN
    const int n_keys_job = min(p.n_keys - kb, p.dma_split_len);  // keys the job may touch

    int limit[2], row[2], head[2];
    bool valid[2];
    int lmax = -1, lmin = 0x7fffffff;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int col = wave * 64 + cb * 32 + l32;
        const int rl = col / p.group;
        row[cb] = tile * p.bm + rl;
        head[cb] = g * p.group + col % p.group;
        valid[cb] = rl < p.bm && row[cb] < p.m;
        limit[cb] = -1;
        if (valid[cb]) {
            limit[cb] = p.row_pos[row[cb]] - kb;   // may be negative: nothing to see here
            lmax = max(lmax, limit[cb]);
            lmin = min(lmin, limit[cb]);
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        lmax = max(lmax, __shfl_xor(lmax, o, 64));
        lmin = min(lmin, __shfl_xor(lmin, o, 64));
    }
    if (lane == 0) s_red[wave] = lmax;
    __syncthreads();
    int tile_max = -1;
#pragma unroll
    for (int w = 0; w < kAttnThreads / 64; ++w) tile_max = max(tile_max, s_red[w]);
    const int key_end = min(tile_max + 1, n_keys_job);
    // (wave-uniform values are moved to scalar registers explicitly: they feed
    // the scalar operands of the global->LDS loads and the loop control)
    const int n_iter = __builtin_amdgcn_readfirstlane((key_end + kBN - 1) / kBN);
    if (n_iter <= 0) {        // block-uniform: no valid row, or no row reaches this range
        if (tid == 0 && p.dma_splits == 1) p.flags[tile * p.hkv + g] = 0;
        continue;
    }
    // sub-steps [0, u_unm) lie entirely at or below every limit of this wave.  A wave
    // without any valid column (the ragged last row tile) has nothing to mask: whatever
    // it computes is dropped, so it takes the cheaper unmasked path throughout.
    const int u_unm = __builtin_amdgcn_readfirstlane(lmin == 0x7fffffff ? 0x3fffffff
                                                                        : (lmin + 1) / 32);

    // ---- Q as B operands -----------------------------------------------------------
    bf16x8 qreg[2][KC];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const bf16_t* qp = p.q + ((int64_t)row[cb] * p.hq + head[cb]) * D + hh * 8;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            if (valid[cb]) {
                qreg[cb][kc] = *reinterpret_cast<const bf16x8*>(qp + kc * 16);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) qreg[cb][kc][e] = (bf16_t)0.0f;
            }
        }
    }

    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};
    f32x16 o_acc[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[db][cb][r] = 0.f;

    // ---- global -> LDS loads ---------------------------------------------------------
    // K stage: row r (key) at byte r*256, logical 16-byte chunk c stored at chunk
    // c ^ (r & 15).  V^T stage: row d at byte d*128, chunk c at c ^ ((d >> 1) & 7).
    // A wave instruction fills 1 KB of LDS: 4 K rows or 8 V^T rows; wave w owns
    // K rows [16w, 16w+16) and V^T rows [32w, 32w+32) of every tile.
    const uint32_t lds_k = (uint32_t)(uintptr_t)smem;
    const uint32_t lds_v = lds_k + NS * kStageK;
    const uint32_t k_row_bytes = (uint32_t)p.hkv * D * 2;
    uint32_t voff_k[4], voff_v[4];
    int krow[4], kchunk16[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 16 * wave + 4 * i + (lane >> 4);
        krow[i] = r;
        kchunk16[i] = (((lane & 15) ^ (r & 15)) * 16);
        voff_k[i] = (uint32_t)r * k_row_bytes + kchunk16[i];
        const int d = 32 * wave + 8 * i + (lane >> 3);
        voff_v[i] = (uint32_t)d * (uint32_t)p.n_pad * 2u + (((lane & 7) ^ ((d >> 1) & 7)) * 16);
    }
    const uint32_t lds_k_wave = __builtin_amdgcn_readfirstlane(lds_k + wave * 16 * 256);
    const uint32_t lds_v_wave = __builtin_amdgcn_readfirstlane(lds_v + wave * 32 * 128);
    const bf16_t* const k_head = p.k + ((int64_t)kb * p.hkv + g) * D;
    const bf16_t* const v_head = p.vt + (int64_t)g * D * p.n_pad + kb;

    // K tile t (clamped to the last tile) into stage st
#define PKV_DMA_K(T, ST)                                                                 \
    {                                                                                    \
        const int t_ = min((T), n_iter - 1);                                             \
        const int t0_ = t_ * kBN;                                                        \
        const bf16_t* gb_ = k_head + (int64_t)t0_ * p.hkv * D;                           \
        const uint32_t lb_ = lds_k_wave + (ST) * kStageK;                                \
        if (t0_ + kBN <= n_keys_job) {                                                   \
            _Pragma("unroll") for (int i = 0; i < 4; ++i)                                \
                dma16(gb_, voff_k[i], lb_ + i * 1024);                                   \
        } else { /* last, ragged tile: rows past the cache re-read its last row */      \
            _Pragma("unroll") for (int i = 0; i < 4; ++i) {                              \
                const int r_ = min(krow[i], n_keys_job - 1 - t0_);                       \
                dma16(gb_, (uint32_t)r_ * k_row_bytes + kchunk16[i], lb_ + i * 1024);    \
            }                                                                            \
        }                                                                                \
    }
#define PKV_DMA_V(T, ST)                                                                 \
    {                                                                                    \
        const int t_ = min((T), n_iter - 1);                                             \
        const bf16_t* gb_ = v_head + t_ * kBN;                                           \
        const uint32_t lb_ = lds_v_wave + (ST) * kStageV;                                \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                    \
            dma16(gb_, voff_v[i], lb_ + i * 1024);                                       \
    }

    // The eight fill instructions of a tile (K tile J+3, V^T tile J+2) go out in four
    // pairs spread over the tile's four scheduling regions: a burst of eight from each
    // of the four waves fills the memory pipeline's queue and stalls the waves.
    // Only the last tile of the cache can be ragged (rows past the cache re-read its last
    // row): its clamped offsets are formed once, every other tile uses the plain ones.
    const bf16_t* gbk_;
    const bf16_t* gbv_;
    bool k_full_;
    uint32_t kofs_last[4];
    {
        const int last_ = (n_keys_job - 1) % kBN;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            kofs_last[i] = (uint32_t)min(krow[i], last_) * k_row_bytes + kchunk16[i];
    }
#define PKV_DMA_PREP(J)                                                                  \
    {                                                                                    \
        const int tk_ = min((J) + 3, n_iter - 1);                                        \
        const int t0k_ = tk_ * kBN;                                                      \
        gbk_ = k_head + (int64_t)t0k_ * p.hkv * D;                                       \
        k_full_ = t0k_ + kBN <= n_keys_job;   /* wave-uniform */                         \
        gbv_ = v_head + min((J) + 2, n_iter - 1) * kBN;                                  \
    }
#define PKV_DMA_PAIR(I, SDK, SDV)                                                        \
    {                                                                                    \
        dma16(gbk_, k_full_ ? voff_k[I] : kofs_last[I],                                  \
              lds_k_wave + (SDK) * kStageK + (I) * 1024);                                \
        dma16(gbv_, voff_v[I], lds_v_wave + (SDV) * kStageV + (I) * 1024);               \
    }

    // ---- LDS -> register operand addresses (bytes inside a stage) ------------------------
    // A-row i of a 32-key block reads key swap_bits23(i) of that block, so that
    // accumulator register r of lane half hh holds key 16*(r/8) + 8*hh + r%8.
    const int prow = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    uint32_t kaddr[KC], vaddr[4];
    {
        const uint32_t a0 = prow * 256 + (((prow & 15) ^ hh) * 16);
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) kaddr[kc] = a0 ^ (kc << 5);
        const uint32_t v0 = l32 * 128 + ((((l32 >> 1) & 7) ^ hh) * 16);
#pragma unroll
        for (int q = 0; q < 4; ++q) vaddr[q] = v0 ^ (q << 5);
    }
    const float c2 = p.scale_log2;

    f32x16 s_a[2], s_b[2];   // S^T of one 32-key sub-step, per column block
    bf16x8 ka[KC], va[2][DB];
    bf16x8 pb[2][2];         // P^T of the current sub-step: [16-key half][column block]
    float rs[2] = {0.f, 0.f};  // this lane's sum of the probabilities being produced
    float msc[2];            // reference maximum times c2 (0 while it is -inf)
    constexpr float kGrow = 1.0e24f;   // ~2^80
    float rs_max = 0.f;
    float e_half = 0.f;      // first probability of the pair being formed
    float x_next;            // exponent of the next score, prepared one step ahead

    // operands of the 32-key half H of the K tile in stage ST
#define PKV_LOAD_KA(ST, H)                                                               \
    _Pragma("unroll") for (int kc = 0; kc < KC; ++kc)                                    \
        ka[kc] = *reinterpret_cast<const bf16x8*>(                                       \
            smem + (ST) * kStageK + (H) * 32 * 256 + kaddr[kc]);
    // V^T operands of the 32-key half H of the tile in stage ST
#define PKV_LOAD_VA(ST, H)                                                               \
    _Pragma("unroll") for (int kk = 0; kk < 2; ++kk)                                     \
    _Pragma("unroll") for (int db = 0; db < DB; ++db)                                    \
        va[kk][db] = *reinterpret_cast<const bf16x8*>(                                   \
            smem + NS * kStageK + (ST) * kStageV + db * 32 * 128 + vaddr[2 * (H) + kk]);

    // The softmax of a sub-step goes one score per MFMA.  p = exp2(s c2 - ref) with the
    // reference of the column block; masked keys give exp2(-inf) = 0.  PKV_SM_PREP
    // forms the exponent of element R of column block CB of score buffer S (first
    // key T0); PKV_SM_STEP turns the exponent prepared one step earlier into the
    // probability of element (CB, R), and prepares the exponent of the next element
    // in between, so that nothing waits on the transcendental unit.  The empty asm
    // statements pin the results where they are computed: without them the compiler
    // sinks the arithmetic towards its uses, away from the MFMAs it should hide under.
#define PKV_SM_PREP(S, CB, R, T0, MASK)                                                  \
    {                                                                                    \
        float x_ = S[CB][R];                                                             \
        if (MASK) {                                                                      \
            const int key_ = (T0) + 16 * ((R) / 8) + 8 * hh + (R) % 8;                   \
            if (key_ > limit[CB]) x_ = -INFINITY;                                        \
        }                                                                                \
        x_next = x_ * c2 - msc[CB];                                                      \
    }
#define PKV_SM_STEP(CB, R, SN, CBN, RN, T0N, MASK)                                       \
    {                                                                                    \
        const float e_ = __builtin_amdgcn_exp2f(x_next);                                 \
        PKV_SM_PREP(SN, CBN, RN, T0N, MASK)                                              \
        rs[CB] += e_;                                                                    \
        if ((R) % 2 == 0) {                                                              \
            e_half = e_;                                                                 \
            asm volatile("" : "+v"(rs[CB]), "+v"(e_half), "+v"(x_next));                 \
        } else {                                                                         \
            pb[(R) / 8][CB][(R) % 8 - 1] = (bf16_t)e_half;                               \
            pb[(R) / 8][CB][(R) % 8] = (bf16_t)e_;                                       \
            asm volatile("" : "+v"(rs[CB]), "+v"(pb[(R) / 8][CB]), "+v"(x_next));        \
        }                                                                                \
    }

    // The reference maximum m_run of a column is NOT the running maximum: it is the
    // maximum of the column's first 32 keys and stays fixed.  The hot loop takes no
    // maximum and never touches the output accumulators with the VALU.  Relative
    // precision does not depend on the reference; what can go wrong is range, when a
    // later score exceeds the reference by more than ~2^80 in the exp2 domain.  So the
    // sums of the probabilities are watched: a partial sum beyond kGrow (or a total
    // that is not finite) marks the tile, and the launcher runs the exact kernel
    // (running maximum, rescaling) on marked tiles afterwards.
#define PKV_ACC(CB)                                                                      \
    {                                                                                    \
        l_run[CB] += rs[CB];                                                             \
        rs_max = fmaxf(rs_max, rs[CB]);                                                  \
        rs[CB] = 0.f;                                                                    \
    }

    // One 32-key sub-step u.  CUR holds S^T(u), NXT receives S^T(u+1) (operands
    // already in ka); (KST, KH) name the K half tile of sub-step u+2, (VST, VH) the
    // V^T half tile of sub-step u; T0 is the first key of sub-step u.  The first
    // four pairs of P(u), column block 0, were formed at the end of sub-step u-1.
    // 32 MFMAs, each pair of them followed by one softmax pair, so that the VALU
    // work is spread evenly under the matrix pipe:
    // (one score after each MFMA):
    //    MFMA  1-16  S^T(u+1)            | P(u): block 0 pairs 4-7, block 1 pairs 0-3
    //    MFMA 17-24  O^T += V^T P^T, b.0 | P(u): block 1 pairs 4-7
    //    MFMA 25-32  O^T += V^T P^T, b.1 | P(u+1): block 0 pairs 0-3
#define PKV_SUBSTEP(CUR, NXT, KST, KH, VST, VH, T0, MASK, DI, SDK, SDV)                  \
    {                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                               \
        PKV_DMA_PAIR(DI, SDK, SDV)                                                       \
        __builtin_amdgcn_sched_barrier(0);                                               \
        PKV_LOAD_VA(VST, VH)                                                             \
        _Pragma("unroll") for (int i_ = 0; i_ < 16; ++i_) {                              \
            const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,                   \
                               0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};                  \
            const int kc_ = i_ >> 1, cbm_ = i_ & 1;                                      \
            NXT[cbm_] = mfma32(ka[kc_], qreg[cbm_][kc_], kc_ == 0 ? z_ : NXT[cbm_]);     \
            if (i_ < 7) { PKV_SM_STEP(0, 8 + i_, CUR, 0, 9 + i_, T0, MASK) }             \
            else if (i_ == 7) { PKV_SM_STEP(0, 15, CUR, 1, 0, T0, MASK) }                \
            else { PKV_SM_STEP(1, i_ - 8, CUR, 1, i_ - 7, T0, MASK) }                    \
            __builtin_amdgcn_sched_barrier(0);                                           \
            if (i_ == 7) {                                                               \
                PKV_ACC(0)                                                               \
                __builtin_amdgcn_sched_barrier(0);                                       \
            }                                                                            \
        }                                                                                \
        PKV_DMA_PAIR((DI) + 1, SDK, SDV)                                                 \
        __builtin_amdgcn_sched_barrier(0);                                               \
        PKV_LOAD_KA(KST, KH)                                                             \
        _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_) {                               \
            const int kk_ = i_ >> 2, db_ = i_ & 3;                                       \
            mfma32_acc(va[kk_][db_], pb[kk_][0], o_acc[db_][0]);                         \
            if (i_ < 7) { PKV_SM_STEP(1, 8 + i_, CUR, 1, 9 + i_, T0, MASK) }             \
            else { PKV_SM_STEP(1, 15, NXT, 0, 0, (T0) + 32, MASK) }                      \
            __builtin_amdgcn_sched_barrier(0);                                           \
        }                                                                                \
        PKV_ACC(1)                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                               \
        _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_) {                               \
            const int kk_ = i_ >> 2, db_ = i_ & 3;                                       \
            mfma32_acc(va[kk_][db_], pb[kk_][1], o_acc[db_][1]);                         \
            PKV_SM_STEP(0, i_, NXT, 0, 1 + i_, (T0) + 32, MASK)                          \
            __builtin_amdgcn_sched_barrier(0);                                           \
        }                                                                                \
    }

    // one 64-key tile J whose V^T sits in stage SV0 and whose successor's K sits in
    // stage SK1; K(J+3) and V^T(J+2) are requested into SDK / SDV
#define PKV_TILE(J, SK1, SV0, SDK, SDV, MASK)                                            \
    {                                                                                    \
        const int t0_tile_ = (J) * kBN;                                                  \
        PKV_DMA_PREP(J)                                                                  \
        PKV_SUBSTEP(s_a, s_b, SK1, 0, SV0, 0, t0_tile_, MASK, 0, SDK, SDV)               \
        PKV_SUBSTEP(s_b, s_a, SK1, 1, SV0, 1, t0_tile_ + 32, MASK, 2, SDK, SDV)          \
        wait_vm<8>();   /* K(J+2), V^T(J+1) have landed; 8 newer loads stay in flight */ \
        __syncthreads();                                                                 \
    }

    // ---- prologue ---------------------------------------------------------------------
    PKV_DMA_K(0, 0)
    PKV_DMA_V(0, 0)
    PKV_DMA_K(1, 1)
    wait_vm<0>();
    __syncthreads();
    PKV_LOAD_KA(0, 0)
    {
        const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                           0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s_a[0] = mfma32(ka[0], qreg[0][0], z_);
        s_a[1] = mfma32(ka[0], qreg[1][0], z_);
#pragma unroll
        for (int kc = 1; kc < KC; ++kc) {
            s_a[0] = mfma32(ka[kc], qreg[0][kc], s_a[0]);
            s_a[1] = mfma32(ka[kc], qreg[1][kc], s_a[1]);
        }
    }
    PKV_LOAD_KA(0, 1)            // operands of S^T(1)
    // first sub-step: nothing accumulated yet, the reference is simply its maximum
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 16 * (r / 8) + 8 * hh + (r % 8);
            if (key <= limit[cb]) mx = fmaxf(mx, s_a[cb][r]);
        }
        m_run[cb] = fmaxf(mx, __shfl_xor(mx, 32, 64));
        msc[cb] = (m_run[cb] == -INFINITY ? 0.f : m_run[cb]) * c2;
    }
    PKV_SM_PREP(s_a, 0, 0, 0, true)
#pragma unroll
    for (int r = 0; r < 8; ++r) PKV_SM_STEP(0, r, s_a, 0, r + 1, 0, true)
    PKV_DMA_K(2, 2)
    PKV_DMA_V(1, 1)

    // ---- main loop: four tiles per trip so that every LDS stage is a constant ------------
    // tile j is mask free when every score it turns into a probability (sub-steps
    // 2j, 2j+1 and the first pairs of 2j+2) lies at or below every limit of the wave:
    // 2j + 2 < u_unm
    int n_unm = min(n_iter, max(0, (u_unm - 1) / 2));
    n_unm &= ~3;
    int j = 0;
    for (; j < n_unm; j += 4) {
        PKV_TILE(j, 1, 0, 3, 2, false)
        PKV_TILE(j + 1, 2, 1, 0, 3, false)
        PKV_TILE(j + 2, 3, 2, 1, 0, false)
        PKV_TILE(j + 3, 0, 3, 2, 1, false)
    }
    for (; j < n_iter; ++j) {
        PKV_TILE(j, (j + 1) & 3, j & 3, (j + 3) & 3, (j + 2) & 3, true)
    }
    wait_vm<0>();   // nothing may still be writing LDS when the workgroup retires
    // the last O^T MFMAs were issued behind the compiler's back: let them retire before
    // the accumulators are read
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

#undef PKV_DMA_K
#undef PKV_DMA_V
#undef PKV_DMA_PREP
#undef PKV_DMA_PAIR
#undef PKV_LOAD_KA
#undef PKV_LOAD_VA
#undef PKV_SM_PREP
#undef PKV_SM_STEP
#undef PKV_ACC
#undef PKV_SUBSTEP
#undef PKV_TILE

    // ---- epilogue ----------------------------------------------------------------------
    float l_tot[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) l_tot[cb] = l_run[cb] + __shfl_xor(l_run[cb], 32, 64);
    {
        const bool bad = !(rs_max < kGrow) || !(l_tot[0] < 3.0e38f) || !(l_tot[1] < 3.0e38f);
        if (__any(bad) && lane == 0) s_red[wave] = 1 << 30;   // s_red held tile limits so far
        else if (lane == 0) s_red[wave] = 0;
        __syncthreads();
        if (tid == 0) {
            const int marked = (s_red[0] | s_red[1] | s_red[2] | s_red[3]) != 0;
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
    // A row whose keys all lie in the first range has its whole result in that range's job:
    // it is written as the final output there and never merged.  Every other row leaves a
    // normalised fp32 partial result per range it reaches.
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        if (!valid[cb]) continue;
        const int pos = min(p.row_pos[row[cb]], p.n_keys - 1);
        const bool direct = p.dma_splits == 1 || pos < p.dma_split_len;
        const float inv = 1.f / l_tot[cb];
        if (!direct) {
            if (pos < kb) continue;   // the row sees nothing of this range
            const int64_t colg = ((int64_t)split * p.m + row[cb]) * p.hq + head[cb];
            float* op = p.part_o + colg * D + 4 * hh;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    f32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = o_acc[db][cb][4 * r4 + e] * inv;
                    *reinterpret_cast<f32x4*>(op + db * 32 + r4 * 8) = v;
                }
            if (hh == 0) p.part_lse[colg] = m_run[cb] * p.scale + logf(l_tot[cb]);
            continue;
        }
        if (split != 0) continue;
        const int64_t colg = (int64_t)row[cb] * p.hq + head[cb];
        bf16_t* op = p.out + colg * D + 4 * hh;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(o_acc[db][cb][4 * r4 + e] * inv);
                *reinterpret_cast<bf16x4*>(op + db * 32 + r4 * 8) = v;
            }
        if (hh == 0) {
            const float lse = m_run[cb] * p.scale + logf(l_tot[cb]);
            if (p.lse) p.lse[colg] = lse;
            // asked for only when every key the row sees is a context key: unsplit launches
            // whose keys are all context keys, and first-range rows (a range boundary lies
            // at the end of the context)
            if (p.lse_ctx) p.lse_ctx[colg] = lse;
        }
    }
  }   // next (kv head, row tile)
}

// Merge of the key ranges of a split launch: out = sum_s w_s O_s / sum_s w_s with
// w_s = exp(lse_s - max lse), over the ranges that begin at or below the row's limit.
// 32 lanes of four output elements per (row, head), eight of them per workgroup.  Rows whose
// keys all lie in the first range were written by that range's job; tiles marked for the
// exact kernel are left to it.
constexpr int kMergeCols = 8;
static_assert(D == 128, "one (row, head) is 32 lanes of four floats");
__global__ __launch_bounds__(32 * kMergeCols) void attn_merge_splits_kernel(AttnParams p) {
    const int64_t col = (int64_t)blockIdx.x * kMergeCols + (threadIdx.x >> 5);   // row * hq + head
    if (col >= (int64_t)p.m * p.hq) return;
    const int row = (int)(col / p.hq), head = (int)(col % p.hq);
    if (p.flags[(row / p.bm) * p.hkv + head / p.group]) return;
    const int limit = min(p.row_pos[row], p.n_keys - 1);
    const int n_s = limit / p.dma_split_len + 1;   // <= dma_splits
    if (n_s == 1) return;
    const int l = threadIdx.x & 31;
    // (unrolled by four so that the loads of four ranges are in flight together: with up to
    // 32 ranges per row the loop is otherwise a chain of memory latencies)
    const float* const lse_col = p.part_lse + (int64_t)row * p.hq + head;
    const float* const o_col = p.part_o + ((int64_t)row * p.hq + head) * D + 4 * l;
    const int64_t lse_step = (int64_t)p.m * p.hq, o_step = lse_step * D;
    float mx = -INFINITY;
#pragma unroll 4
    for (int sp = 0; sp < n_s; ++sp) mx = fmaxf(mx, lse_col[sp * lse_step]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float wsum = 0.f;
#pragma unroll 4
    for (int sp = 0; sp < n_s; ++sp) {
        const float w = __expf(lse_col[sp * lse_step] - mx);
        const f32x4 o = *reinterpret_cast<const f32x4*>(o_col + sp * o_step);
        wsum += w;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += w * o[e];
    }
    bf16x4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(acc[e] / wsum);
    *reinterpret_cast<bf16x4*>(p.out + col * D + 4 * l) = v;
    if (p.lse && l == 0) p.lse[col] = mx + logf(wsum);
    if (p.lse_ctx && l == 0) {
        // the ranges that lie below ctx_keys (a range boundary): the same sum, cut there
        const int n_c = min(n_s, p.ctx_keys / p.dma_split_len);
        float mc = -INFINITY;
        for (int sp = 0; sp < n_c; ++sp)
            mc = fmaxf(mc, p.part_lse[((int64_t)sp * p.m + row) * p.hq + head]);
        float wc = 0.f;
        for (int sp = 0; sp < n_c; ++sp)
            wc += __expf(p.part_lse[((int64_t)sp * p.m + row) * p.hq + head] - mc);
        p.lse_ctx[col] = mc + logf(wc);
    }
}

}  // namespace

namespace {
// 8 (default) or 4 waves per workgroup, from PKV_ATTN_WAVES, read once
int attn_main_waves() {
    static std::atomic<int> waves{0};
    int nw = waves.load(std::memory_order_relaxed);
    if (nw == 0) {
        const char* e = std::getenv("PKV_ATTN_WAVES");
        nw = (e && e[0] == '4') ? 4 : 8;
        waves.store(nw, std::memory_order_relaxed);
    }
    return nw;
}
}  // namespace

int attn_dma128_v_source() {
    if (attn_main_waves() != 8) return 1;
    // read at every call, so that one process can run both sources side by side
    const char* e = std::getenv("PKV_ATTN_VT");
    return !e ? -1 : (e[0] == '1' ? 1 : (e[0] == '0' ? 0 : -1));
}

pkv_status launch_attn_dma128(const AttnParams& p, hipStream_t st) {
    // every workgroup reports through p.flags; the operands must all be there
    if (!p.q || !p.k || !p.vt || !p.row_pos || !p.out || !p.flags || !p.queue)
        return PKV_ERR_NULL;
    if (p.v && attn_main_waves() != 8) return PKV_ERR_UNSUPPORTED;
    if (p.dma_splits < 1 || p.dma_split_len < kBN || p.dma_split_len % kBN ||
        (int64_t)p.dma_splits * p.dma_split_len < p.n_keys)
        return PKV_ERR_SHAPE;
    if (p.dma_splits > 1 && (!p.part_o || !p.part_lse)) return PKV_ERR_WORKSPACE;
    static std::atomic<bool> configured{false};   // set twice at worst: the calls are idempotent
    if (!configured.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(attn_dma128_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess)
            return PKV_ERR_LAUNCH;
        configured.store(true, std::memory_order_release);
    }
    static std::atomic<int> n_cu_cached{0};   // per process; the devices of one machine are alike
    int n_cu = n_cu_cached.load(std::memory_order_relaxed);
    if (n_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            v <= 0)
            return PKV_ERR_LAUNCH;
        n_cu = v;
        n_cu_cached.store(v, std::memory_order_relaxed);
    }
    // Two kernels do this job: eight waves of 32 columns (two waves per SIMD, the default)
    // and four waves of 64 columns (one per SIMD).  PKV_ATTN_WAVES=4 in the environment
    // selects the latter, for comparisons.
    const int nw = attn_main_waves();
    if (nw == 8) {
        const pkv_status rc = launch_attn_w8_main(p, n_cu, st);
        if (rc != PKV_OK) return rc;
    } else {
        // one workgroup per CU (its LDS admits no second one), or per tile if there are fewer
        const int64_t grid = std::min<int64_t>((int64_t)p.n_tiles * p.dma_splits * p.hkv, n_cu);
        hipLaunchKernelGGL(attn_dma128_kernel, dim3((unsigned)grid), dim3(kAttnThreads),
                           kLdsBytes, st, p);
        if (launch_status() != PKV_OK) return PKV_ERR_LAUNCH;
    }
    if (p.dma_splits > 1)
        hipLaunchKernelGGL(attn_merge_splits_kernel,
                           dim3((unsigned)(((int64_t)p.m * p.hq + kMergeCols - 1) / kMergeCols)),
                           dim3(32 * kMergeCols), 0, st, p);
    return launch_status();
}

}  // namespace pkv
