// Step 5: causal attention of the recomputed rows (selected context tokens
// and user-query tokens) over the whole updated cache.
// (Paper: Sec. 4.3 Stage II, complete recomputation but only for the
// selected tokens; Sec. 5.3, this attention dominates the cost; Eq. 1.)
//
//   out[i,h] = sum_{t <= row_pos[i]} softmax_t(q[i,h] . K[t,g(h)] * scale) V[t,g(h)]
#include "pkv_common.h"

namespace pkv {

namespace {

// ---------------------------------------------------------------------------
// Generic kernel: any head_dim (multiple of 16, <= 256), fp32 or bf16
// storage, plain fp32 FMAs.  One block per (row, head).  Keys are walked in
// tiles of blockDim keys: thread j scores key j of the tile, the tile maximum
// updates the running maximum (online softmax), then thread c accumulates
// output element c over the tile's values (coalesced along head_dim).
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void sparse_row_attn_generic(
    const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc,
    const int32_t* __restrict__ row_pos, T* __restrict__ out,
    float* __restrict__ lse_out, int hq, int hkv, int d, float scale) {
    constexpr int V = Vec16<T>::N;
    typedef typename Vec16<T>::type vec_t;
    __shared__ float qs[256];
    __shared__ float ps[256];
    __shared__ float red[4];
    __shared__ float s_m;
    const int i = blockIdx.x;
    const int h = blockIdx.y;
    const int g = h / (hq / hkv);
    const int tid = threadIdx.x;
    const int nthr = blockDim.x;
    const int last = row_pos[i];
    const T* qrow = q + ((int64_t)i * hq + h) * d;
    if (tid < d) qs[tid] = Elem<T>::load(qrow + tid);
    __syncthreads();
    float m = -INFINITY, l = 0.f, acc = 0.f;
    for (int t0 = 0; t0 <= last; t0 += nthr) {
        const int t = t0 + tid;
        float s = -INFINITY;
        if (t <= last) {
            const T* krow = kc + ((int64_t)t * hkv + g) * d;
            float a = 0.f;
            for (int c = 0; c < d; c += V) {
                const vec_t kv = *reinterpret_cast<const vec_t*>(krow + c);
#pragma unroll
                for (int j = 0; j < V; ++j) a += qs[c + j] * Elem<T>::to_f32(kv[j]);
            }
            s = a * scale;
        }
        // tile maximum
        float tm = s;
        for (int o = 32; o > 0; o >>= 1) tm = fmaxf(tm, __shfl_xor(tm, o, 64));
        if ((tid & 63) == 0) red[tid >> 6] = tm;
        __syncthreads();
        if (tid == 0) {
            float x = red[0];
            for (int w = 1; w < (nthr >> 6); ++w) x = fmaxf(x, red[w]);
            s_m = fmaxf(m, x);
        }
        __syncthreads();
        const float mn = s_m;  // finite: key t0 is always visible
        const float corr = expf(m - mn);
        const float p = t <= last ? expf(s - mn) : 0.f;
        ps[tid] = p;
        // tile sum of p
        float ts = p;
        for (int o = 32; o > 0; o >>= 1) ts += __shfl_xor(ts, o, 64);
        __syncthreads();  // ps visible; red free again
        if ((tid & 63) == 0) red[tid >> 6] = ts;
        __syncthreads();
        float tsum = 0.f;
        for (int w = 0; w < (nthr >> 6); ++w) tsum += red[w];
        l = l * corr + tsum;
        m = mn;
        if (tid < d) {
            acc *= corr;
            const int cnt = last - t0 + 1 < nthr ? last - t0 + 1 : nthr;
            const T* vbase = vc + ((int64_t)t0 * hkv + g) * d + tid;
            for (int j = 0; j < cnt; ++j)
                acc += ps[j] * Elem<T>::load(vbase + (int64_t)j * hkv * d);
        }
        __syncthreads();  // before ps / red are overwritten
    }
    if (tid < d) out[((int64_t)i * hq + h) * d + tid] = Elem<T>::from_f32(acc / l);
    if (lse_out && tid == 0) lse_out[(int64_t)i * hq + h] = m + logf(l);
}

}  // namespace

size_t sparse_row_attn_ws_bytes(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m) {
    (void)cfg; (void)n_keys; (void)m;
    return 0;
}

pkv_status launch_sparse_row_attn(const pkv_layer_cfg& cfg, const void* q,
                                  const void* k_cache, const void* v_cache,
                                  const int32_t* row_pos, void* out,
                                  float* lse_out, int64_t m, int64_t n_keys,
                                  float scale, void* ws, hipStream_t st) {
    (void)ws; (void)n_keys;
    if (m == 0) return PKV_OK;
    const int d = cfg.head_dim;
    const int block = d <= 64 ? 64 : (d <= 128 ? 128 : 256);
    const dim3 grid((unsigned)m, (unsigned)cfg.n_q_heads);
    if (cfg.dtype == PKV_BF16) {
        hipLaunchKernelGGL(sparse_row_attn_generic<bf16_t>, grid, dim3(block), 0, st,
                           (const bf16_t*)q, (const bf16_t*)k_cache,
                           (const bf16_t*)v_cache, row_pos, (bf16_t*)out, lse_out,
                           cfg.n_q_heads, cfg.n_kv_heads, d, scale);
    } else {
        hipLaunchKernelGGL(sparse_row_attn_generic<float>, grid, dim3(block), 0, st,
                           (const float*)q, (const float*)k_cache,
                           (const float*)v_cache, row_pos, (float*)out, lse_out,
                           cfg.n_q_heads, cfg.n_kv_heads, d, scale);
    }
    return launch_status();
}

}  // namespace pkv
