// Step 2: query-driven value function.
// (Paper: Algorithm 1 first stage, alpha_l = Softmax(Q_s K'^T / sqrt(d_k));
// Sec. 4.2, mean over the user-query tokens; Appendix E, mean over heads;
// Algorithm 1 second stage, the per-layer scores are summed.)
//
//   score[t] (+)= 1/(Hq nq) sum_{h,q} exp(s[h,q,t] - lse[h,q]),
//   s = q . k * scale,  lse[h,q] = log sum_t exp(s[h,q,t])
//
// Two passes over the keys, because the normaliser of a query column must be
// known before its probabilities can be summed down the columns:
//   pass 1  lse per (query token, head) column;
//   pass 2  per key, the sum over all columns of exp(s - lse), written once
//           per key (no atomics, so the result is deterministic).
#include "score_common.h"

namespace pkv {

namespace {

// ---------------------------------------------------------------------------
// Generic kernels: any head_dim (multiple of 16), any group size, fp32 or
// bf16 storage, plain fp32 FMA arithmetic.
// ---------------------------------------------------------------------------

template <typename T>
__device__ __forceinline__ float dot_row(const float* __restrict__ qs,
                                         const T* __restrict__ krow, int d) {
    constexpr int V = Vec16<T>::N;
    typedef typename Vec16<T>::type vec_t;
    float acc = 0.f;
    for (int c = 0; c < d; c += V) {
        const vec_t kv = *reinterpret_cast<const vec_t*>(krow + c);
#pragma unroll
        for (int j = 0; j < V; ++j) acc += qs[c + j] * Elem<T>::to_f32(kv[j]);
    }
    return acc;
}

// pass 1: one block per (query token, head) column
template <typename T>
__global__ __launch_bounds__(256) void score_lse_generic(
    const T* __restrict__ q, const T* __restrict__ k, float* __restrict__ lse,
    int n_ctx, int hq, int hkv, int d, float scale) {
    __shared__ float qs[256];
    __shared__ float red_m[4], red_l[4];
    const int col = blockIdx.x;  // = qi * hq + h
    const int h = col % hq;
    const int g = h / (hq / hkv);
    const int tid = threadIdx.x;
    if (tid < d) qs[tid] = Elem<T>::load(q + (int64_t)col * d + tid);
    __syncthreads();
    float m = -INFINITY, l = 0.f;
    for (int t = tid; t < n_ctx; t += 256) {
        const float s = dot_row<T>(qs, k + ((int64_t)t * hkv + g) * d, d) * scale;
        const float mn = fmaxf(m, s);
        l = l * expf(m - mn) + expf(s - mn);
        m = mn;
    }
    // wave reduce, then across the 4 waves
    for (int o = 32; o > 0; o >>= 1) {
        const float mo = __shfl_xor(m, o, 64);
        const float lo = __shfl_xor(l, o, 64);
        const float mn = fmaxf(m, mo);
        const float a = m == -INFINITY ? 0.f : l * expf(m - mn);
        const float b = mo == -INFINITY ? 0.f : lo * expf(mo - mn);
        l = a + b;
        m = mn;
    }
    if ((tid & 63) == 0) {
        red_m[tid >> 6] = m;
        red_l[tid >> 6] = l;
    }
    __syncthreads();
    if (tid == 0) {
        float mm = red_m[0], ll = red_l[0];
        for (int w = 1; w < 4; ++w) {
            const float mn = fmaxf(mm, red_m[w]);
            const float a = mm == -INFINITY ? 0.f : ll * expf(mm - mn);
            const float b = red_m[w] == -INFINITY ? 0.f : red_l[w] * expf(red_m[w] - mn);
            ll = a + b;
            mm = mn;
        }
        lse[col] = mm + logf(ll);
    }
}

// pass 2: one thread per key, all kv heads and all columns in sequence
template <typename T>
__global__ __launch_bounds__(256) void score_colsum_generic(
    const T* __restrict__ q, const T* __restrict__ k,
    const float* __restrict__ lse, float* __restrict__ score, int nq, int n_ctx,
    int hq, int hkv, int d, float scale, int accumulate,
    const int32_t* __restrict__ row_pos = nullptr) {
    __shared__ float qs[256];
    const int t = blockIdx.x * 256 + threadIdx.x;
    float sum = 0.f;
    const int ncol = nq * hq;
    for (int col = 0; col < ncol; ++col) {
        __syncthreads();
        if (threadIdx.x < d) qs[threadIdx.x] = Elem<T>::load(q + (int64_t)col * d + threadIdx.x);
        __syncthreads();
        // with row limits a query row only counts for the keys it sees
        if (t < n_ctx && (!row_pos || t <= row_pos[col / hq])) {
            const int g = (col % hq) / (hq / hkv);
            const float s = dot_row<T>(qs, k + ((int64_t)t * hkv + g) * d, d) * scale;
            sum += expf(s - lse[col]);
        }
    }
    if (t < n_ctx) {
        const float a = sum / (float)ncol;
        score[t] = accumulate ? score[t] + a : a;
    }
}


// ---------------------------------------------------------------------------
// MFMA path: bf16 storage, head_dim 64 or 128, group size <= 16.
//
// Pass 1 reuses the attention kernel of step 5 with its PV half switched off:
// it yields per-column (max, sum) partials over splits of the key range, which
// merge_lse_kernel folds into one log2-domain normaliser per column.
//
// Pass 2 (below): a workgroup owns 256 keys of one kv head (64 per wave, held
// in registers as MFMA A operands for the whole kernel) and walks over all
// columns (query token, head of the group) in blocks of 32:
//     S^T [64 keys x 32 cols] = K (A, registers) x Q^T (B, from L1/L2)
//     acc[key] += exp2(S^T * c - lse2[col])
// The accumulator of lane l holds column l%32, so the running per-key sums
// stay in registers and are reduced across the 32 lanes once, at the end.
// Each (kv head, key) partial is written exactly once; finish_score_kernel adds
// the kv heads in a fixed order, so the score is deterministic.
// ---------------------------------------------------------------------------

// 64 columns per block; the four waves fold every fourth split each, then meet in LDS
__global__ __launch_bounds__(256) void merge_lse_kernel(const float* __restrict__ part_ml,
                                                        float* __restrict__ lse2, int ncol,
                                                        int n_splits, float scale_log2) {
    __shared__ float s_m[4][64], s_l[4][64];
    const int c = threadIdx.x & 63, part = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + c;
    float mx = -INFINITY, sum = 0.f;
    if (col < ncol) {
        for (int s = part; s < n_splits; s += 4) {
            const float2 ml = *reinterpret_cast<const float2*>(part_ml + ((int64_t)s * ncol + col) * 2);
            if (ml.x == -INFINITY) continue;
            const float mn = fmaxf(mx, ml.x);
            sum = sum * exp2f((mx - mn) * scale_log2) + ml.y * exp2f((ml.x - mn) * scale_log2);
            mx = mn;
        }
    }
    s_m[part][c] = mx;
    s_l[part][c] = sum;
    __syncthreads();
    if (part == 0 && col < ncol) {
        float m = -INFINITY;
        for (int q = 0; q < 4; ++q) m = fmaxf(m, s_m[q][c]);
        float l = 0.f;
        for (int q = 0; q < 4; ++q)
            if (s_m[q][c] != -INFINITY) l += s_l[q][c] * exp2f((s_m[q][c] - m) * scale_log2);
        lse2[col] = m * scale_log2 + log2f(l);
    }
}

// kCausal: row_pos[query row] is the last key that row sees; column blocks that see
// nothing of this wave's keys are skipped, the others are masked per key.
template <int D, bool kCausal = false>
__global__ __launch_bounds__(256) void score_colsum_mfma(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const float* __restrict__ lse2, float* __restrict__ part_score, int nq, int n_ctx,
    int hq, int hkv, int group, float scale_log2,
    const int32_t* __restrict__ row_pos = nullptr) {
    constexpr int KC = D / 16;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int hh = lane >> 5, l32 = lane & 31;
    const int g = blockIdx.y;
    const int key0 = blockIdx.x * 256 + wave * 64;

    bf16x8 a[2][KC];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        const int key = min(key0 + 32 * kb + l32, n_ctx - 1);
        const bf16_t* kp = k + ((int64_t)key * hkv + g) * D + hh * 8;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
            a[kb][kc] = *reinterpret_cast<const bf16x8*>(kp + kc * 16);
    }
    f32x16 acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[kb][r] = 0.f;

    const int ncol_g = nq * group;
    // operands of column block c0 (clamped: lanes past the last column re-read it and
    // are switched off through an infinite normaliser)
    bf16x8 b[KC], bn[KC];
    float norm, norm_n;
    int lim = 0x7fffffff, lim_n = 0x7fffffff;   // last key the lane's column sees
    auto load_cols = [&](int c0, bf16x8* dst, float* nrm, int* limit) {
        const int col = min(c0 + l32, ncol_g - 1);
        const int qi = col / group;
        const int h = g * group + col % group;
        const bf16_t* qp = q + ((int64_t)qi * hq + h) * D + hh * 8;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) dst[kc] = *reinterpret_cast<const bf16x8*>(qp + kc * 16);
        *nrm = c0 + l32 < ncol_g ? lse2[(int64_t)qi * hq + h] : INFINITY;
        if (kCausal) *limit = c0 + l32 < ncol_g ? row_pos[qi] : -1;
    };
    load_cols(0, b, &norm, &lim);
    for (int c0 = 0; c0 < ncol_g; c0 += 32) {
        // next block, in flight during the MFMAs
        load_cols(min(c0 + 32, ncol_g - 1), bn, &norm_n, &lim_n);
        if (kCausal && __ballot(lim >= key0) == 0) {   // nobody here sees these keys
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) b[kc] = bn[kc];
            norm = norm_n;
            lim = lim_n;
            continue;
        }
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][kc], b[kc], s[0], 0, 0, 0);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][kc], b[kc], s[1], 0, 0, 0);
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float e = __builtin_amdgcn_exp2f(s[kb][r] * scale_log2 - norm);
                if (kCausal) {
                    const int key = key0 + 32 * kb + 8 * (r / 4) + 4 * hh + (r % 4);
                    acc[kb][r] += key <= lim ? e : 0.f;
                } else {
                    acc[kb][r] += e;
                }
            }
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) b[kc] = bn[kc];
        norm = norm_n;
        lim = lim_n;
    }
    // sum over the 32 columns held by the lanes of each half
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v = acc[kb][r];
            for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            acc[kb][r] = v;
        }
    if (l32 == 0) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + 32 * kb + 8 * (r / 4) + 4 * hh + (r % 4);
                if (key < n_ctx) part_score[(int64_t)g * n_ctx + key] = acc[kb][r];
            }
    }
}

// 64 keys per block; the four waves add every fourth partial each (in order), then
// meet in LDS in a fixed order: deterministic
__global__ __launch_bounds__(256) void finish_score_kernel(const float* __restrict__ part_score,
                                                           float* __restrict__ score, int n_ctx,
                                                           int n_parts, float inv_ncol,
                                                           int accumulate) {
    __shared__ float s_part[4][64];
    const int kx = threadIdx.x & 63, py = threadIdx.x >> 6;
    const int t = blockIdx.x * 64 + kx;
    float s = 0.f;
    if (t < n_ctx)
        for (int q = py; q < n_parts; q += 4) s += part_score[(int64_t)q * n_ctx + t];
    s_part[py][kx] = s;
    __syncthreads();
    if (py == 0 && t < n_ctx) {
        const float tot = ((s_part[0][kx] + s_part[1][kx]) + s_part[2][kx]) + s_part[3][kx];
        score[t] = accumulate ? score[t] + tot * inv_ncol : tot * inv_ncol;
    }
}

// natural-log normalisers (what the attention call emits) -> the log2-domain ones the
// column-sum kernels subtract
__global__ __launch_bounds__(256) void lse_to_log2_kernel(const float* __restrict__ lse,
                                                          float* __restrict__ lse2, int ncol) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < ncol) lse2[i] = lse[i] * 1.4426950408889634f;
}

bool mfma_score_supported(const pkv_layer_cfg& cfg) {
    const int group = cfg.n_q_heads / cfg.n_kv_heads;
    return cfg.dtype == PKV_BF16 && (cfg.head_dim == 64 || cfg.head_dim == 128) &&
           group <= 16;
}

struct SplitPlan {
    int n_splits, split_len;
};

SplitPlan plan_splits(const pkv_layer_cfg& cfg, int64_t n_ctx, int64_t nq) {
    const int group = cfg.n_q_heads / cfg.n_kv_heads;
    const int64_t tiles = ceil_div(nq, 256 / group) * cfg.n_kv_heads;
    int64_t want = ceil_div(1024, tiles);
    const int64_t max_splits = ceil_div(n_ctx, 256);
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    int64_t len = ceil_div(ceil_div(n_ctx, want), 64) * 64;
    SplitPlan sp;
    sp.split_len = (int)len;
    sp.n_splits = (int)ceil_div(n_ctx, len);
    return sp;
}

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

pkv_status launch_attn_lse_partials(const pkv_layer_cfg& cfg, const void* q,
                                    const void* k, int64_t nq, int64_t n_ctx,
                                    float scale, int n_splits, int split_len,
                                    float* part_ml, hipStream_t st);

size_t query_score_ws_bytes(const pkv_layer_cfg& cfg, int64_t n_ctx, int64_t nq) {
    const size_t ncol = (size_t)(nq * cfg.n_q_heads);
    if (!mfma_score_supported(cfg)) return ncol * sizeof(float);
    // the key-blocked kernels (other geometries, and the column sums with row limits)
    const SplitPlan sp = plan_splits(cfg, n_ctx, nq);
    size_t need = align_up(ncol * sizeof(float)) +
                  align_up((size_t)sp.n_splits * ncol * 2 * sizeof(float)) +
                  align_up((size_t)cfg.n_kv_heads * n_ctx * sizeof(float));
    if (score_dma128_supported(cfg, n_ctx, nq)) {
        const ScorePlan dp = plan_score_dma128(cfg, n_ctx, nq);
        const size_t dma = align_up(ncol * sizeof(float)) +
                           align_up((size_t)dp.n_splits * ncol * 2 * sizeof(float)) +
                           align_up((size_t)dp.n_parts * n_ctx * sizeof(float));
        if (dma > need) need = dma;
    }
    return need;
}

pkv_status launch_query_score(const pkv_layer_cfg& cfg, const void* q,
                              const void* k, float* score, int64_t nq,
                              int64_t n_ctx, float scale, int accumulate,
                              void* ws, hipStream_t st) {
    float* lse = (float*)ws;
    const int ncol = (int)(nq * cfg.n_q_heads);
    const int hq = cfg.n_q_heads, hkv = cfg.n_kv_heads, d = cfg.head_dim;
    if (mfma_score_supported(cfg) && score_dma128_supported(cfg, n_ctx, nq)) {
        const ScorePlan sp = plan_score_dma128(cfg, n_ctx, nq);
        unsigned char* base = (unsigned char*)ws;
        float* lse2 = (float*)base;
        float* part_ml = (float*)(base + align_up((size_t)ncol * sizeof(float)));
        float* part_score = (float*)((unsigned char*)part_ml +
                                     align_up((size_t)sp.n_splits * ncol * 2 * sizeof(float)));
        ScoreParams sp_ = {};
        sp_.q = (const bf16_t*)q;
        sp_.k = (const bf16_t*)k;
        sp_.part_ml = part_ml;
        sp_.lse2 = lse2;
        sp_.lse_factor = 1.0f;   // merge_lse_kernel writes log2-domain values
        sp_.part_score = part_score;
        sp_.nq = (int)nq; sp_.n_ctx = (int)n_ctx; sp_.hq = hq; sp_.hkv = hkv; sp_.group = hq / hkv;
        sp_.n_cblk = sp.n_cblk; sp_.n_splits = sp.n_splits; sp_.split_len = sp.split_len;
        sp_.scale_log2 = scale * 1.4426950408889634f;
        pkv_status stt = launch_score_dma128(1, sp_, st);
        if (stt != PKV_OK) return stt;
        hipLaunchKernelGGL(merge_lse_kernel, dim3((unsigned)ceil_div(ncol, 64)), dim3(256),
                           0, st, part_ml, lse2, ncol, sp.n_splits, sp_.scale_log2);
        stt = launch_score_dma128(2, sp_, st);
        if (stt != PKV_OK) return stt;
        hipLaunchKernelGGL(finish_score_kernel, dim3((unsigned)ceil_div(n_ctx, 64)),
                           dim3(256), 0, st, part_score, score, (int)n_ctx, sp.n_parts,
                           1.0f / (float)ncol, accumulate);
        return launch_status();
    }
    if (mfma_score_supported(cfg)) {
        const SplitPlan sp = plan_splits(cfg, n_ctx, nq);
        unsigned char* base = (unsigned char*)ws;
        float* lse2 = (float*)base;
        float* part_ml = (float*)(base + align_up((size_t)ncol * sizeof(float)));
        float* part_score = (float*)((unsigned char*)part_ml +
                                     align_up((size_t)sp.n_splits * ncol * 2 * sizeof(float)));
        const float scale_log2 = scale * 1.4426950408889634f;
        pkv_status stt = launch_attn_lse_partials(cfg, q, k, nq, n_ctx, scale, sp.n_splits,
                                                  sp.split_len, part_ml, st);
        if (stt != PKV_OK) return stt;
        hipLaunchKernelGGL(merge_lse_kernel, dim3((unsigned)ceil_div(ncol, 64)), dim3(256),
                           0, st, part_ml, lse2, ncol, sp.n_splits, scale_log2);
        const dim3 grid((unsigned)ceil_div(n_ctx, 256), (unsigned)hkv);
        if (d == 128) {
            hipLaunchKernelGGL(score_colsum_mfma<128>, grid, dim3(256), 0, st,
                               (const bf16_t*)q, (const bf16_t*)k, lse2, part_score,
                               (int)nq, (int)n_ctx, hq, hkv, hq / hkv, scale_log2);
        } else {
            hipLaunchKernelGGL(score_colsum_mfma<64>, grid, dim3(256), 0, st,
                               (const bf16_t*)q, (const bf16_t*)k, lse2, part_score,
                               (int)nq, (int)n_ctx, hq, hkv, hq / hkv, scale_log2);
        }
        hipLaunchKernelGGL(finish_score_kernel, dim3((unsigned)ceil_div(n_ctx, 64)),
                           dim3(256), 0, st, part_score, score, (int)n_ctx, hkv,
                           1.0f / (float)ncol, accumulate);
        return launch_status();
    }
    const unsigned kb = (unsigned)ceil_div(n_ctx, 256);
    if (cfg.dtype == PKV_BF16) {
        hipLaunchKernelGGL(score_lse_generic<bf16_t>, dim3(ncol), dim3(256), 0, st,
                           (const bf16_t*)q, (const bf16_t*)k, lse, (int)n_ctx, hq,
                           hkv, d, scale);
        hipLaunchKernelGGL(score_colsum_generic<bf16_t>, dim3(kb), dim3(256), 0, st,
                           (const bf16_t*)q, (const bf16_t*)k, lse, score, (int)nq,
                           (int)n_ctx, hq, hkv, d, scale, accumulate);
    } else {
        hipLaunchKernelGGL(score_lse_generic<float>, dim3(ncol), dim3(256), 0, st,
                           (const float*)q, (const float*)k, lse, (int)n_ctx, hq,
                           hkv, d, scale);
        hipLaunchKernelGGL(score_colsum_generic<float>, dim3(kb), dim3(256), 0, st,
                           (const float*)q, (const float*)k, lse, score, (int)nq,
                           (int)n_ctx, hq, hkv, d, scale, accumulate);
    }
    return launch_status();
}

// Column sums with normalisers supplied by the caller (one key stream instead of two).
// row_pos == nullptr: every query row counts for every key, the fast kernels run.
// row_pos != nullptr: query row i counts for keys <= row_pos[i] only.
pkv_status launch_query_score_lse(const pkv_layer_cfg& cfg, const void* q, const void* k,
                                  const float* lse, const int32_t* row_pos, float* score,
                                  int64_t nq, int64_t n_ctx, float scale, int accumulate,
                                  void* ws, hipStream_t st) {
    const int ncol = (int)(nq * cfg.n_q_heads);
    const int hq = cfg.n_q_heads, hkv = cfg.n_kv_heads, d = cfg.head_dim;
    const float scale_log2 = scale * 1.4426950408889634f;
    if (!mfma_score_supported(cfg)) {
        const unsigned kb = (unsigned)ceil_div(n_ctx, 256);
        if (cfg.dtype == PKV_BF16)
            hipLaunchKernelGGL(score_colsum_generic<bf16_t>, dim3(kb), dim3(256), 0, st,
                               (const bf16_t*)q, (const bf16_t*)k, lse, score, (int)nq,
                               (int)n_ctx, hq, hkv, d, scale, accumulate, row_pos);
        else
            hipLaunchKernelGGL(score_colsum_generic<float>, dim3(kb), dim3(256), 0, st,
                               (const float*)q, (const float*)k, lse, score, (int)nq,
                               (int)n_ctx, hq, hkv, d, scale, accumulate, row_pos);
        return launch_status();
    }
    // workspace layout of launch_query_score: normalisers first, the partial column sums
    // behind the (unused here) partial normalisers
    unsigned char* base = (unsigned char*)ws;
    float* lse2 = (float*)base;
    if (!row_pos && score_dma128_supported(cfg, n_ctx, nq)) {
        const ScorePlan sp = plan_score_dma128(cfg, n_ctx, nq);
        float* part_score = (float*)(base + align_up((size_t)ncol * sizeof(float)) +
                                     align_up((size_t)sp.n_splits * ncol * 2 * sizeof(float)));
        ScoreParams sp_ = {};
        sp_.q = (const bf16_t*)q;
        sp_.k = (const bf16_t*)k;
        sp_.lse2 = lse;   // natural log: the kernel converts as it loads
        sp_.lse_factor = 1.4426950408889634f;
        sp_.part_score = part_score;
        sp_.nq = (int)nq; sp_.n_ctx = (int)n_ctx; sp_.hq = hq; sp_.hkv = hkv; sp_.group = hq / hkv;
        sp_.n_cblk = sp.n_cblk; sp_.n_splits = sp.n_splits; sp_.split_len = sp.split_len;
        sp_.scale_log2 = scale_log2;
        const pkv_status stt = launch_score_dma128(2, sp_, st);
        if (stt != PKV_OK) return stt;
        hipLaunchKernelGGL(finish_score_kernel, dim3((unsigned)ceil_div(n_ctx, 64)),
                           dim3(256), 0, st, part_score, score, (int)n_ctx, sp.n_parts,
                           1.0f / (float)ncol, accumulate);
        return launch_status();
    }
    hipLaunchKernelGGL(lse_to_log2_kernel, dim3((unsigned)ceil_div(ncol, 256)), dim3(256), 0,
                       st, lse, lse2, ncol);
    const SplitPlan sp = plan_splits(cfg, n_ctx, nq);
    float* part_score = (float*)(base + align_up((size_t)ncol * sizeof(float)) +
                                 align_up((size_t)sp.n_splits * ncol * 2 * sizeof(float)));
    const dim3 grid((unsigned)ceil_div(n_ctx, 256), (unsigned)hkv);
#define PKV_COLSUM(DD, CAUSAL)                                                              \
    hipLaunchKernelGGL((score_colsum_mfma<DD, CAUSAL>), grid, dim3(256), 0, st,             \
                       (const bf16_t*)q, (const bf16_t*)k, lse2, part_score, (int)nq,       \
                       (int)n_ctx, hq, hkv, hq / hkv, scale_log2, row_pos)
    if (d == 128) {
        if (row_pos) PKV_COLSUM(128, true); else PKV_COLSUM(128, false);
    } else {
        if (row_pos) PKV_COLSUM(64, true); else PKV_COLSUM(64, false);
    }
#undef PKV_COLSUM
    hipLaunchKernelGGL(finish_score_kernel, dim3((unsigned)ceil_div(n_ctx, 64)), dim3(256), 0,
                       st, part_score, score, (int)n_ctx, hkv, 1.0f / (float)ncol, accumulate);
    return launch_status();
}

}  // namespace pkv
