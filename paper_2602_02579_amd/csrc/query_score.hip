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
#include "pkv_common.h"

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
    int hq, int hkv, int d, float scale, int accumulate) {
    __shared__ float qs[256];
    const int t = blockIdx.x * 256 + threadIdx.x;
    float sum = 0.f;
    const int ncol = nq * hq;
    for (int col = 0; col < ncol; ++col) {
        __syncthreads();
        if (threadIdx.x < d) qs[threadIdx.x] = Elem<T>::load(q + (int64_t)col * d + threadIdx.x);
        __syncthreads();
        if (t < n_ctx) {
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

}  // namespace

size_t query_score_ws_bytes(const pkv_layer_cfg& cfg, int64_t n_ctx, int64_t nq) {
    (void)n_ctx;
    return (size_t)(nq * cfg.n_q_heads) * sizeof(float);
}

pkv_status launch_query_score(const pkv_layer_cfg& cfg, const void* q,
                              const void* k, float* score, int64_t nq,
                              int64_t n_ctx, float scale, int accumulate,
                              void* ws, hipStream_t st) {
    float* lse = (float*)ws;
    const int ncol = (int)(nq * cfg.n_q_heads);
    const int hq = cfg.n_q_heads, hkv = cfg.n_kv_heads, d = cfg.head_dim;
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

}  // namespace pkv
