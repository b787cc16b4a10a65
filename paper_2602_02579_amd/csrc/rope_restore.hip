// Step 1: rotary position restore on the assembled, position-free keys.
// (Paper: Sec. 1 footnote on position-independent key caches; Appendix E:
// positions go onto the old key cache once, before cache replacement.)
//
// HBM-bound streaming kernel.  One work item owns, for one token, a 16-byte
// run of pair indices i (8 bf16 or 4 fp32) and walks over all kv heads, so
// the sin/cos of a (token, i) pair is computed once and reused by every
// head.  Consecutive lanes own consecutive 16-byte runs, so a wave reads
// whole 128-byte (bf16, D=128) half-head segments of consecutive tokens.
#include "pkv_common.h"

#include <cmath>

namespace pkv {

void fill_rope_table(RopeTable* t, int head_dim, double theta) {
    const int half = head_dim / 2;
    for (int i = 0; i < kMaxHalfDim; ++i)
        t->inv_freq[i] = i < half ? std::pow(theta, -2.0 * i / head_dim) : 0.0;
}

template <typename T>
__global__ __launch_bounds__(256) void rope_restore_kernel(
    const T* k_in, T* k_out,
    const int32_t* __restrict__ pos, int64_t pos_base, int64_t n, int n_heads,
    int head_dim, RopeTable tab) {
    constexpr int V = Vec16<T>::N;
    typedef typename Vec16<T>::type vec_t;
    const int half = head_dim / 2;
    const int chunks = half / V;  // work items per token
    const int64_t total = n * chunks;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total;
         w += stride) {
        const int64_t t = w / chunks;
        const int i0 = (int)(w - t * chunks) * V;
        const double p = pos ? (double)pos[t] : (double)(pos_base + t);
        const T* src = k_in + t * (int64_t)n_heads * head_dim + i0;
        T* dst = k_out + t * (int64_t)n_heads * head_dim + i0;
        // heads in batches of HB: all loads of a batch are issued before its
        // stores, which keeps many 16-byte requests in flight per lane without
        // assuming that k_in and k_out do not alias (in place is allowed); the
        // first batch is requested before the sines and cosines are worked out,
        // so that arithmetic runs under the memory latency
        constexpr int HB = 8;
        vec_t a[HB], b[HB];
        auto load_batch = [&](int h0) {
#pragma unroll
            for (int u = 0; u < HB; ++u) {
                if (h0 + u < n_heads) {
                    // streamed once: non-temporal, so that the lines do not displace what the
                    // caches hold for the kernels around this one
                    a[u] = __builtin_nontemporal_load(
                        reinterpret_cast<const vec_t*>(src + (h0 + u) * head_dim));
                    b[u] = __builtin_nontemporal_load(
                        reinterpret_cast<const vec_t*>(src + (h0 + u) * head_dim + half));
                }
            }
        };
        load_batch(0);
        float sn[V], cs[V];
#pragma unroll
        for (int j = 0; j < V; ++j) rope_sincos(p, tab.inv_freq[i0 + j], &sn[j], &cs[j]);
        for (int h0 = 0; h0 < n_heads; h0 += HB) {
            if (h0 > 0) load_batch(h0);
#pragma unroll
            for (int u = 0; u < HB; ++u) {
                if (h0 + u < n_heads) {
                    vec_t ra, rb;
#pragma unroll
                    for (int j = 0; j < V; ++j) {
                        const float x = Elem<T>::to_f32(a[u][j]);
                        const float y = Elem<T>::to_f32(b[u][j]);
                        ra[j] = Elem<T>::from_f32(x * cs[j] - y * sn[j]);
                        rb[j] = Elem<T>::from_f32(y * cs[j] + x * sn[j]);
                    }
                    __builtin_nontemporal_store(ra, reinterpret_cast<vec_t*>(dst + (h0 + u) * head_dim));
                    __builtin_nontemporal_store(
                        rb, reinterpret_cast<vec_t*>(dst + (h0 + u) * head_dim + half));
                }
            }
        }
    }
}

pkv_status launch_rope_restore(const pkv_layer_cfg& cfg, const void* k_in,
                               void* k_out, const int32_t* pos,
                               int64_t pos_base, int64_t n, hipStream_t st) {
    if (n == 0) return PKV_OK;
    RopeTable tab;
    fill_rope_table(&tab, cfg.head_dim, (double)cfg.rope_theta);
    const int half = cfg.head_dim / 2;
    const int v = cfg.dtype == PKV_BF16 ? 8 : 4;
    const int64_t total = n * (half / v);
    const int block = 256;
    int64_t grid = ceil_div(total, block);
    if (grid > 256 * 64) grid = 256 * 64;  // grid-stride beyond 64 blocks per CU
    if (cfg.dtype == PKV_BF16) {
        hipLaunchKernelGGL(rope_restore_kernel<bf16_t>, dim3((unsigned)grid),
                           dim3(block), 0, st, (const bf16_t*)k_in,
                           (bf16_t*)k_out, pos, pos_base, n, cfg.n_kv_heads,
                           cfg.head_dim, tab);
    } else {
        hipLaunchKernelGGL(rope_restore_kernel<float>, dim3((unsigned)grid),
                           dim3(block), 0, st, (const float*)k_in,
                           (float*)k_out, pos, pos_base, n, cfg.n_kv_heads,
                           cfg.head_dim, tab);
    }
    return launch_status();
}

}  // namespace pkv
