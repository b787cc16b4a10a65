// Step 3: top-p selection - indices of the k largest fused scores, ties to
// the lower index, returned in ascending index order.
// (Paper: Eq. 4, TOP_p of the value function; Algorithm 1, "Select token
// indices"; Sec. 4.3: the set is chosen once and used by every layer.)
//
// One workgroup of 1024 lanes (16 waves).  The score vector is small (128 KB
// at 32k context) and stays in L2, so the kernel is latency-bound.
//
// Up to 64 scores per lane (n <= 65536) the keys live in registers, each lane
// owning a contiguous run of indices (topk_bisect_kernel):
//   1. the key tau of the k-th largest score is built bit by bit from the top:
//      up to 32 rounds of "how many keys are >= candidate" (it stops at the round
//      that leaves exactly k keys), each a compare-and-count
//      over the lane's registers, a DPP row reduction and one barrier - no
//      atomics, so the skewed digit distribution of real scores (all in two or
//      three binades) costs nothing;
//   2. two block-wide exclusive scans (keys > tau, keys == tau) give every
//      lane the output offset of its run; equal keys are taken in index order
//      until the need is met - the lower-index tie rule.
// Longer vectors use the radix kernel below:
//   1. radix select, 4 passes of 8 bits over order-preserving uint32 keys,
//      finds the key tau of the k-th largest score and how many scores equal
//      to tau are still needed;
//   2. an index-ordered compaction: every wave owns a contiguous segment,
//      counts its (> tau, == tau) elements with ballots, a 16-entry scan
//      gives each wave its output offset, and a second walk writes the
//      selected indices.  An element equal to tau is taken only while the
//      number of equal elements at lower indices is below the need, which is
//      exactly the lower-index tie rule.
#include "pkv_common.h"

namespace pkv {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;

// larger float <=> larger key; -0.0 is folded onto +0.0 first
__device__ __forceinline__ uint32_t order_key(float x) {
    uint32_t u = __float_as_uint(x + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t lanemask_lt() {
    const int lane = threadIdx.x & 63;
    return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

__global__ __launch_bounds__(kThreads) void topk_select_kernel(
    const float* __restrict__ score, int n, int k, int32_t* __restrict__ idx_out) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_prefix, s_remaining;
    __shared__ uint32_t wave_gt[kWaves], wave_eq[kWaves], wave_off[kWaves],
        wave_eq_before[kWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // ---- 1. radix select of the k-th largest key --------------------------
    if (tid == 0) {
        s_prefix = 0;
        s_remaining = (uint32_t)k;
    }
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
        for (int i = tid; i < n; i += kThreads) {
            const uint32_t key = order_key(score[i]);
            if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns digits 4l .. 4l+3; suffix sums from the top digit
            uint32_t c[4];
            uint32_t mine = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = hist[4 * lane + j];
                mine += c[j];
            }
            // inclusive suffix scan over lanes (higher lanes = larger digits)
            uint32_t suf = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t o = __shfl_down(suf, d, 64);
                if (lane + d < 64) suf += o;
            }
            uint32_t above = suf - mine;  // elements with digits above my four
            const uint32_t remaining = s_remaining;
            // digits from high to low inside my four
#pragma unroll
            for (int j = 3; j >= 0; --j) {
                if (above < remaining && remaining <= above + c[j]) {
                    s_prefix = prefix | ((uint32_t)(4 * lane + j) << shift);
                    s_remaining = remaining - above;
                }
                above += c[j];
            }
        }
        __syncthreads();
    }
    const uint32_t tau = s_prefix;
    const uint32_t need = s_remaining;  // elements == tau still to take (>= 1 if k > 0)

    // ---- 2. index-ordered compaction ---------------------------------------
    int seg = (n + kWaves - 1) / kWaves;
    seg = (seg + 63) & ~63;
    const int begin = wave * seg < n ? wave * seg : n;
    const int end = begin + seg < n ? begin + seg : n;

    uint32_t gt = 0, eq = 0;
    for (int i = begin + lane; i - lane < end; i += 64) {
        const bool in = i < end;
        const uint32_t key = in ? order_key(score[i]) : 0u;
        gt += __popcll(__ballot(in && key > tau));
        eq += __popcll(__ballot(in && key == tau));
    }
    if (lane == 0) {
        wave_gt[wave] = gt;
        wave_eq[wave] = eq;
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t off = 0, eqb = 0;
        for (int w = 0; w < kWaves; ++w) {
            wave_off[w] = off;
            wave_eq_before[w] = eqb;
            const uint32_t room = eqb < need ? need - eqb : 0u;
            off += wave_gt[w] + (wave_eq[w] < room ? wave_eq[w] : room);
            eqb += wave_eq[w];
        }
    }
    __syncthreads();
    if (k == 0) return;
    uint32_t out = wave_off[wave];
    uint32_t eq_run = wave_eq_before[wave];
    const uint64_t lt = lanemask_lt();
    for (int i = begin + lane; i - lane < end; i += 64) {
        const bool in = i < end;
        const uint32_t key = in ? order_key(score[i]) : 0u;
        const uint64_t beq = __ballot(in && key == tau);
        const bool is_eq = in && key == tau;
        const bool take = in && (key > tau ||
                                 (is_eq && eq_run + __popcll(beq & lt) < need));
        const uint64_t bsel = __ballot(take);
        if (take) idx_out[out + __popcll(bsel & lt)] = i;
        out += __popcll(bsel);
        eq_run += __popcll(beq);
    }
}

// sum over the wave of a small per-lane count, returned wave-uniform
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
    // inclusive scan inside each row of 16 lanes (row_shr 1, 2, 4, 8; lanes shifted in
    // from outside the row read 0), then the four row totals
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 15) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 31) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 47) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

template <int ITEMS>
__global__ __launch_bounds__(kThreads) void topk_bisect_kernel(
    const float* __restrict__ score, int n, int k, int32_t* __restrict__ idx_out) {
    __shared__ uint32_t s_wave[2][kWaves];
    __shared__ uint32_t s_scan[2][kWaves];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // lane tid owns indices [tid * ITEMS, tid * ITEMS + ITEMS); indices >= n get key 0,
    // which is below the key of every float (order_key(-inf) = 0x007fffff)
    uint32_t key[ITEMS];
    const int base = tid * ITEMS;
#pragma unroll
    for (int j = 0; j < ITEMS; j += 4) {
        if (base + j + 3 < n) {
            const float4 v = *reinterpret_cast<const float4*>(score + base + j);
            key[j] = order_key(v.x);
            key[j + 1] = order_key(v.y);
            key[j + 2] = order_key(v.z);
            key[j + 3] = order_key(v.w);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                key[j + e] = base + j + e < n ? order_key(score[base + j + e]) : 0u;
        }
    }

    // block-wide count of keys for which PRED holds (one barrier; s_wave is double
    // buffered so that a fast wave cannot overwrite what a slow one still reads)
    int round = 0;
#define PKV_BLOCK_COUNT(PRED, RESULT)                                                    \
    {                                                                                    \
        uint32_t c_ = 0;                                                                 \
        _Pragma("unroll") for (int j = 0; j < ITEMS; ++j) c_ += (PRED) ? 1u : 0u;        \
        c_ = wave_sum(c_);                                                               \
        if (lane == 0) s_wave[round & 1][wave] = c_;                                     \
        __syncthreads();                                                                 \
        uint32_t t_ = 0;                                                                 \
        _Pragma("unroll") for (int w = 0; w < kWaves; ++w) t_ += s_wave[round & 1][w];   \
        RESULT = t_;                                                                     \
        ++round;                                                                         \
    }

    // ---- 1. tau = the k-th largest key, bit by bit ---------------------------------
    uint32_t tau = 0;
    for (int b = 31; b >= 0; --b) {
        const uint32_t cand = tau | (1u << b);
        uint32_t cnt;
        PKV_BLOCK_COUNT(key[j] >= cand, cnt)
        if (cnt >= (uint32_t)k) tau = cand;
        // exactly k keys at or above the candidate: they are the selection, the lower bits
        // of the k-th key do not matter (block-uniform; with distinct scores this happens
        // at the highest bit in which the k-th and the (k+1)-th key differ)
        if (cnt == (uint32_t)k) break;
    }
    uint32_t n_gt;
    PKV_BLOCK_COUNT(key[j] > tau, n_gt)
    const uint32_t need = (uint32_t)k - n_gt;   // keys == tau still to take
#undef PKV_BLOCK_COUNT

    // ---- 2. output offsets: exclusive scans over the lanes in index order -------------
    uint32_t my_gt = 0, my_eq = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        my_gt += key[j] > tau ? 1u : 0u;
        my_eq += key[j] == tau ? 1u : 0u;
    }
    uint32_t in_gt = my_gt, in_eq = my_eq;   // inclusive scans inside the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t og = __shfl_up(in_gt, d, 64), oe = __shfl_up(in_eq, d, 64);
        if (lane >= d) {
            in_gt += og;
            in_eq += oe;
        }
    }
    if (lane == 63) {
        s_scan[0][wave] = in_gt;
        s_scan[1][wave] = in_eq;
    }
    __syncthreads();
    uint32_t gt_before = in_gt - my_gt, eq_before = in_eq - my_eq;
    for (int w = 0; w < wave; ++w) {
        gt_before += s_scan[0][w];
        eq_before += s_scan[1][w];
    }
    // equal keys at lower indices are taken first, until `need` of them are
    uint32_t out = gt_before + (eq_before < need ? eq_before : need);
    uint32_t eq_seen = eq_before;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const bool is_eq = key[j] == tau;
        const bool take = key[j] > tau || (is_eq && eq_seen < need);
        if (take) idx_out[out++] = base + j;
        eq_seen += is_eq ? 1u : 0u;
    }
}

}  // namespace

pkv_status launch_topk_select(const float* score, int64_t n, int64_t k,
                              int32_t* idx_out, hipStream_t st) {
    if (n == 0 || k == 0) return PKV_OK;
    // the register kernels read 16 bytes at a time
    const bool aligned = (reinterpret_cast<uintptr_t>(score) & 15) == 0;
    // a round costs one vector compare-and-count per register key, so short vectors take
    // the instantiation with the fewest keys per lane that holds them
    if (aligned && n <= 8 * kThreads) {
        hipLaunchKernelGGL(topk_bisect_kernel<8>, dim3(1), dim3(kThreads), 0, st, score,
                           (int)n, (int)k, idx_out);
        return launch_status();
    }
    if (aligned && n <= 16 * kThreads) {
        hipLaunchKernelGGL(topk_bisect_kernel<16>, dim3(1), dim3(kThreads), 0, st, score,
                           (int)n, (int)k, idx_out);
        return launch_status();
    }
    if (aligned && n <= 32 * kThreads) {
        hipLaunchKernelGGL(topk_bisect_kernel<32>, dim3(1), dim3(kThreads), 0, st, score,
                           (int)n, (int)k, idx_out);
        return launch_status();
    }
    if (aligned && n <= 64 * kThreads) {
        hipLaunchKernelGGL(topk_bisect_kernel<64>, dim3(1), dim3(kThreads), 0, st, score,
                           (int)n, (int)k, idx_out);
        return launch_status();
    }
    hipLaunchKernelGGL(topk_select_kernel, dim3(1), dim3(kThreads), 0, st, score,
                       (int)n, (int)k, idx_out);
    return launch_status();
}

}  // namespace pkv
