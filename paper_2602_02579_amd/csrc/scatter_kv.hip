// Step 4b: cache update - recomputed K/V rows replace the cache rows they
// belong to; every other row is left as it is.
// (Paper: Algorithm 1, "Update layer-wise KV cache" and the user-query K/V.)
//
// Pure data movement: a row is Hkv*D elements (2 KB for bf16 Llama-3-8B
// geometry), copied as 16-byte pieces by consecutive lanes, so every wave
// moves whole contiguous kilobytes.  blockIdx.y picks K or V.
#include "pkv_common.h"

namespace pkv {

__global__ __launch_bounds__(256) void scatter_rows_kernel(
    const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
    const int32_t* __restrict__ dst_row, uint4* __restrict__ k_cache,
    uint4* __restrict__ v_cache, int64_t m, int vec_per_row) {
    const uint4* src = blockIdx.y ? v_new : k_new;
    uint4* dst = blockIdx.y ? v_cache : k_cache;
    const int64_t total = m * vec_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total;
         w += stride) {
        const int64_t i = w / vec_per_row;
        const int c = (int)(w - i * vec_per_row);
        dst[(int64_t)dst_row[i] * vec_per_row + c] = src[w];
    }
}

// rows of a power-of-two number of 16-byte pieces (the usual case: 128 for bf16
// Llama-3-8B geometry): no division, two pieces per lane in flight
__global__ __launch_bounds__(256) void scatter_rows_pow2_kernel(
    const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
    const int32_t* __restrict__ dst_row, uint4* __restrict__ k_cache,
    uint4* __restrict__ v_cache, int64_t m, int log2_vec) {
    const uint4* src = blockIdx.y ? v_new : k_new;
    uint4* dst = blockIdx.y ? v_cache : k_cache;
    const int64_t total = m << log2_vec;
    const int64_t w0 = (int64_t)blockIdx.x * 512 + threadIdx.x;
    const int64_t w1 = w0 + 256;
    const int64_t mask = ((int64_t)1 << log2_vec) - 1;
    uint4 a, b;
    int64_t da = 0, db = 0;
    if (w0 < total) {
        da = ((int64_t)dst_row[w0 >> log2_vec] << log2_vec) + (w0 & mask);
        a = src[w0];
    }
    if (w1 < total) {
        db = ((int64_t)dst_row[w1 >> log2_vec] << log2_vec) + (w1 & mask);
        b = src[w1];
    }
    if (w0 < total) dst[da] = a;
    if (w1 < total) dst[db] = b;
}

pkv_status launch_scatter_kv(const pkv_layer_cfg& cfg, const void* k_new,
                             const void* v_new, const int32_t* dst_row,
                             void* k_cache, void* v_cache, int64_t m,
                             hipStream_t st) {
    if (m == 0) return PKV_OK;
    const int elt = cfg.dtype == PKV_BF16 ? 2 : 4;
    const int vec_per_row = cfg.n_kv_heads * cfg.head_dim * elt / 16;
    const int64_t total = m * vec_per_row;
    if ((vec_per_row & (vec_per_row - 1)) == 0 && ceil_div(total, 512) < (1 << 30)) {
        int log2_vec = 0;
        while ((1 << log2_vec) < vec_per_row) ++log2_vec;
        hipLaunchKernelGGL(scatter_rows_pow2_kernel,
                           dim3((unsigned)ceil_div(total, 512), 2), dim3(256), 0, st,
                           (const uint4*)k_new, (const uint4*)v_new, dst_row,
                           (uint4*)k_cache, (uint4*)v_cache, m, log2_vec);
        return launch_status();
    }
    int64_t grid = ceil_div(total, 256);
    if (grid > 256 * 32) grid = 256 * 32;
    hipLaunchKernelGGL(scatter_rows_kernel, dim3((unsigned)grid, 2), dim3(256),
                       0, st, (const uint4*)k_new, (const uint4*)v_new, dst_row,
                       (uint4*)k_cache, (uint4*)v_cache, m, vec_per_row);
    return launch_status();
}

}  // namespace pkv
