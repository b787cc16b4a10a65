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


// ---------------------------------------------------------------------------
// Longer vectors (n > 24576) with a workspace: the same radix select spread over many
// workgroups, so that the counting runs at the bandwidth of the whole chip instead of one
// CU's.  A workgroup of 256 lanes owns 2048 consecutive scores (8 per lane, in registers).
//   hist<0>  histogram of the top 11 key bits              -> hist0[2048]
//   hist<1>  (bin0, rest0) from hist0; next 11 bits of the keys in bin0 -> hist1[2048]
//   hist<2>  (bin1, rest1) from hist1; last 10 bits of the keys in (bin0, bin1) -> hist2[1024]
//   count    (bin2, need) from hist2 gives tau; per workgroup (keys > tau, keys == tau)
//   write    exclusive sums over the workgroups before mine give my output offset; equal
//            keys are taken in index order until `need` of them are - the lower-index rule
// Each kernel scans only the newest histogram: workgroup 0 leaves the (bin, rest) pair it
// found in the workspace for the kernels behind it.  Histogram updates are integer
// atomics, so the result does not depend on their order.
// Workspace (uint32 words): hist0[2048] hist1[2048] hist2[1024] sel[8] counts[2 * n_wg].
// ---------------------------------------------------------------------------
constexpr int kSeg = 2048;          // scores per workgroup
constexpr int kSegThreads = 256;
constexpr int kHistWords = 2048 + 2048 + 1024;

__global__ __launch_bounds__(256) void topk_ws_zero_kernel(uint32_t* __restrict__ ws) {
    for (int i = threadIdx.x; i < kHistWords + 8; i += 256) ws[i] = 0u;
}

// The bin b (counted from the top) with count(bins > b) < rest <= count(bins >= b), and what
// is left of rest inside it.  All 256 lanes call it; the result is block-uniform.
__device__ __forceinline__ void topk_find_bin(const uint32_t* __restrict__ hist, int nbins,
                                              uint32_t rest, uint32_t* bin_out,
                                              uint32_t* rest_out) {
    __shared__ uint32_t s_wsum[4];
    __shared__ uint32_t s_res[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = nbins / kSegThreads;          // 8 or 4
    uint32_t c[8];
    uint32_t mine = 0;
    // lane t owns bins [nbins - (t + 1) per, nbins - t per): the top bins belong to lane 0
    const int hi = nbins - tid * per;
    for (int j = 0; j < per; ++j) {
        c[j] = hist[hi - 1 - j];                  // descending
        mine += c[j];
    }
    uint32_t inc = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) s_wsum[wave] = inc;
    __syncthreads();
    uint32_t above = inc - mine;                  // keys in bins above mine
    for (int w = 0; w < wave; ++w) above += s_wsum[w];
    for (int j = 0; j < per; ++j) {
        if (above < rest && rest <= above + c[j]) {
            s_res[0] = (uint32_t)(hi - 1 - j);
            s_res[1] = rest - above;
        }
        above += c[j];
    }
    __syncthreads();
    *bin_out = s_res[0];
    *rest_out = s_res[1];
    __syncthreads();                              // s_res / s_wsum may be reused
}

__device__ __forceinline__ void topk_load_keys(const float* __restrict__ score, int n, int base,
                                               bool aligned, uint32_t* key) {
#pragma unroll
    for (int j = 0; j < 8; j += 4) {
        if (aligned && base + j + 3 < n) {
            const float4 v = *reinterpret_cast<const float4*>(score + base + j);
            key[j] = order_key(v.x);
            key[j + 1] = order_key(v.y);
            key[j + 2] = order_key(v.z);
            key[j + 3] = order_key(v.w);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)   // indices >= n: key 0, below every float's key
                key[j + e] = base + j + e < n ? order_key(score[base + j + e]) : 0u;
        }
    }
}

template <int PASS>
__global__ __launch_bounds__(256) void topk_ws_hist_kernel(const float* __restrict__ score, int n,
                                                           int k, uint32_t* __restrict__ ws,
                                                           int aligned) {
    __shared__ uint32_t s_hist[2048];
    uint32_t* hist0 = ws;
    uint32_t* hist1 = ws + 2048;
    uint32_t* hist2 = ws + 4096;
    uint32_t* sel = ws + kHistWords;
    const int tid = threadIdx.x;
    constexpr int nbins = PASS == 2 ? 1024 : 2048;
    for (int i = tid; i < nbins; i += 256) s_hist[i] = 0u;
    uint32_t prefix = 0;        // the key bits fixed so far, right-aligned
    if (PASS == 1) {
        uint32_t b, r;
        topk_find_bin(hist0, 2048, (uint32_t)k, &b, &r);
        if (blockIdx.x == 0 && tid == 0) { sel[0] = b; sel[1] = r; }
        prefix = b;
    } else if (PASS == 2) {
        uint32_t b, r;
        topk_find_bin(hist1, 2048, sel[1], &b, &r);
        if (blockIdx.x == 0 && tid == 0) { sel[2] = b; sel[3] = r; }
        prefix = (sel[0] << 11) | b;
    } else {
        __syncthreads();
    }
    uint32_t key[8];
    const int base = blockIdx.x * kSeg + tid * 8;
    topk_load_keys(score, n, base, aligned != 0, key);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (base + j >= n) continue;
        if (PASS == 0) atomicAdd(&s_hist[key[j] >> 21], 1u);
        else if (PASS == 1) { if ((key[j] >> 21) == prefix) atomicAdd(&s_hist[(key[j] >> 10) & 2047u], 1u); }
        else { if ((key[j] >> 10) == prefix) atomicAdd(&s_hist[key[j] & 1023u], 1u); }
    }
    __syncthreads();
    uint32_t* out = PASS == 0 ? hist0 : PASS == 1 ? hist1 : hist2;
    for (int i = tid; i < nbins; i += 256)
        if (s_hist[i]) atomicAdd(&out[i], s_hist[i]);
}

__global__ __launch_bounds__(256) void topk_ws_count_kernel(const float* __restrict__ score, int n,
                                                            uint32_t* __restrict__ ws, int aligned) {
    __shared__ uint32_t s_g[4], s_e[4];
    uint32_t* hist2 = ws + 4096;
    uint32_t* sel = ws + kHistWords;
    uint32_t* counts = sel + 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t b, need;
    topk_find_bin(hist2, 1024, sel[3], &b, &need);
    if (blockIdx.x == 0 && tid == 0) { sel[4] = b; sel[5] = need; }
    const uint32_t tau = (sel[0] << 21) | (sel[2] << 10) | b;
    uint32_t key[8];
    const int base = blockIdx.x * kSeg + tid * 8;
    topk_load_keys(score, n, base, aligned != 0, key);
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        gt += key[j] > tau ? 1u : 0u;
        eq += (key[j] == tau && base + j < n) ? 1u : 0u;
    }
    for (int o = 32; o > 0; o >>= 1) {
        gt += __shfl_xor(gt, o, 64);
        eq += __shfl_xor(eq, o, 64);
    }
    if (lane == 0) { s_g[wave] = gt; s_e[wave] = eq; }
    __syncthreads();
    if (tid == 0) {
        counts[2 * blockIdx.x] = s_g[0] + s_g[1] + s_g[2] + s_g[3];
        counts[2 * blockIdx.x + 1] = s_e[0] + s_e[1] + s_e[2] + s_e[3];
    }
}

__global__ __launch_bounds__(256) void topk_ws_write_kernel(const float* __restrict__ score, int n,
                                                            const uint32_t* __restrict__ ws,
                                                            int32_t* __restrict__ idx_out,
                                                            int aligned) {
    __shared__ uint32_t s_g[4], s_e[4];
    const uint32_t* sel = ws + kHistWords;
    const uint32_t* counts = sel + 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t tau = (sel[0] << 21) | (sel[2] << 10) | sel[4];
    const uint32_t need = sel[5];
    // keys > tau and keys == tau in the workgroups before mine
    uint32_t gb = 0, eb = 0;
    for (int w = tid; w < (int)blockIdx.x; w += 256) {
        gb += counts[2 * w];
        eb += counts[2 * w + 1];
    }
    for (int o = 32; o > 0; o >>= 1) {
        gb += __shfl_xor(gb, o, 64);
        eb += __shfl_xor(eb, o, 64);
    }
    if (lane == 0) { s_g[wave] = gb; s_e[wave] = eb; }
    __syncthreads();
    const uint32_t gt_wg = s_g[0] + s_g[1] + s_g[2] + s_g[3];
    const uint32_t eq_wg = s_e[0] + s_e[1] + s_e[2] + s_e[3];
    __syncthreads();
    uint32_t key[8];
    const int base = blockIdx.x * kSeg + tid * 8;
    topk_load_keys(score, n, base, aligned != 0, key);
    uint32_t my_gt = 0, my_eq = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        my_gt += key[j] > tau ? 1u : 0u;
        my_eq += (key[j] == tau && base + j < n) ? 1u : 0u;
    }
    uint32_t in_gt = my_gt, in_eq = my_eq;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t og = __shfl_up(in_gt, d, 64), oe = __shfl_up(in_eq, d, 64);
        if (lane >= d) { in_gt += og; in_eq += oe; }
    }
    if (lane == 63) { s_g[wave] = in_gt; s_e[wave] = in_eq; }
    __syncthreads();
    uint32_t gt_before = gt_wg + in_gt - my_gt, eq_before = eq_wg + in_eq - my_eq;
    for (int w = 0; w < wave; ++w) {
        gt_before += s_g[w];
        eq_before += s_e[w];
    }
    // equal keys at lower indices are taken first, until `need` of them are
    uint32_t out = gt_before + (eq_before < need ? eq_before : need);
    uint32_t eq_seen = eq_before;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const bool is_eq = key[j] == tau && base + j < n;
        const bool take = key[j] > tau || (is_eq && eq_seen < need);
        if (take) idx_out[out++] = base + j;
        eq_seen += is_eq ? 1u : 0u;
    }
}

}  // namespace

// Shortest vector that takes the many-workgroup kernels when a workspace is given: their six
// launches cost a flat ~20 us, the one-workgroup register kernel 10 us at 4k scores, 16 us
// at 16k, 29 us at 32k and 46 us at 64k.
constexpr int64_t kWsMin = 24 * 1024 + 1;

size_t topk_select_ws_bytes(int64_t n) {
    if (n < kWsMin || n > ((int64_t)1 << 22)) return 0;   // other kernels, no scratch
    return (size_t)(kHistWords + 8 + 2 * ceil_div(n, kSeg)) * sizeof(uint32_t);
}

pkv_status launch_topk_select(const float* score, int64_t n, int64_t k,
                              int32_t* idx_out, void* ws, size_t ws_bytes, hipStream_t st) {
    if (n == 0 || k == 0) return PKV_OK;
    // the register kernels read 16 bytes at a time
    const bool aligned = (reinterpret_cast<uintptr_t>(score) & 15) == 0;
    const size_t need = topk_select_ws_bytes(n);
    if (need && ws && ws_bytes >= need && (reinterpret_cast<uintptr_t>(ws) & 3) == 0) {
        uint32_t* w = (uint32_t*)ws;
        const dim3 grid((unsigned)ceil_div(n, kSeg)), block(kSegThreads);
        const int al = aligned ? 1 : 0;
        hipLaunchKernelGGL(topk_ws_zero_kernel, dim3(1), block, 0, st, w);
        hipLaunchKernelGGL(topk_ws_hist_kernel<0>, grid, block, 0, st, score, (int)n, (int)k, w, al);
        hipLaunchKernelGGL(topk_ws_hist_kernel<1>, grid, block, 0, st, score, (int)n, (int)k, w, al);
        hipLaunchKernelGGL(topk_ws_hist_kernel<2>, grid, block, 0, st, score, (int)n, (int)k, w, al);
        hipLaunchKernelGGL(topk_ws_count_kernel, grid, block, 0, st, score, (int)n, w, al);
        hipLaunchKernelGGL(topk_ws_write_kernel, grid, block, 0, st, score, (int)n, w, idx_out, al);
        return launch_status();
    }
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
    // no (or too small a) workspace: one workgroup does it all
    hipLaunchKernelGGL(topk_select_kernel, dim3(1), dim3(kThreads), 0, st, score,
                       (int)n, (int)k, idx_out);
    return launch_status();
}

}  // namespace pkv
