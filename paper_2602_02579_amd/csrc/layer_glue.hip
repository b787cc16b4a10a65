// The rest of a pre-norm decoder layer for the rows that are carried through the model
// (paper: Sec. 4.2, the user query against the imprecise cache; Sec. 4.3 and Appendix E,
// the selected and the query rows through every layer): RMS normalisation of gathered
// rows, a linear layer with an optional residual, and the gated up-projection of the
// MLP.  The block is the public Llama one; the paper does not restate it.
//
// bf16 linear layers of MFMA-friendly sizes run on the 256 x 256 tile kernel of the
// Q/K/V projection with a different epilogue (gather_qkv_proj_dma.hip); everything else
// (fp32, odd sizes, unaligned pointers) takes the simple kernels below, one wave per
// output element.
#include "proj_common.h"

namespace pkv {

namespace {

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// ---- RMS normalisation: one wave per row, 16 bytes per lane and step ---------------
// The row is read twice (sum of squares, then scaling); the second read comes out of
// the cache.  Rows of up to 8 steps per lane (8 KB: hidden 4096 in bf16) stay in
// registers instead.
template <typename T, bool IN_REGS>
__global__ __launch_bounds__(256) void rmsnorm_rows_kernel(const T* __restrict__ h,
                                                           const int32_t* __restrict__ row_idx,
                                                           const T* __restrict__ weight,
                                                           float eps, T* __restrict__ y,
                                                           int m, int hidden) {
    typedef typename Vec16<T>::type vec_t;
    constexpr int N = Vec16<T>::N;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= m) return;
    const int64_t src = row_idx ? row_idx[row] : row;
    const vec_t* hp = reinterpret_cast<const vec_t*>(h + src * hidden);
    const vec_t* wp = reinterpret_cast<const vec_t*>(weight);
    vec_t* yp = reinterpret_cast<vec_t*>(y + (int64_t)row * hidden);
    const int n_chunks = hidden / N;
    float ss = 0.f;
    if (IN_REGS) {
        vec_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = i * 64 + lane;
            if (c < n_chunks) {
                v[i] = __builtin_nontemporal_load(hp + c);   // every row is read once
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    const float f = Elem<T>::to_f32(v[i][e]);
                    ss += f * f;
                }
            }
        }
        ss = wave_sum_f32(ss);
        const float r = 1.0f / sqrtf(ss / (float)hidden + eps);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = i * 64 + lane;
            if (c < n_chunks) {
                const vec_t w = wp[c];
                vec_t o;
#pragma unroll
                for (int e = 0; e < N; ++e)
                    o[e] = Elem<T>::from_f32(Elem<T>::to_f32(v[i][e]) * r * Elem<T>::to_f32(w[e]));
                __builtin_nontemporal_store(o, yp + c);
            }
        }
    } else {
        for (int c = lane; c < n_chunks; c += 64) {
            const vec_t v = hp[c];
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const float f = Elem<T>::to_f32(v[e]);
                ss += f * f;
            }
        }
        ss = wave_sum_f32(ss);
        const float r = 1.0f / sqrtf(ss / (float)hidden + eps);
        for (int c = lane; c < n_chunks; c += 64) {
            const vec_t v = hp[c];
            const vec_t w = wp[c];
            vec_t o;
#pragma unroll
            for (int e = 0; e < N; ++e)
                o[e] = Elem<T>::from_f32(Elem<T>::to_f32(v[e]) * r * Elem<T>::to_f32(w[e]));
            yp[c] = o;
        }
    }
}

// ---- row gather: 16 bytes per lane ------------------------------------------------------
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ src,
                                                          const int32_t* __restrict__ row_idx,
                                                          uint4* __restrict__ dst, int64_t total,
                                                          int chunks) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int64_t row = i / chunks;
    const int c = (int)(i - row * chunks);
    dst[i] = src[(int64_t)row_idx[row] * chunks + c];
}

// ---- simple linear layers: one wave per output element ----------------------------------
template <typename T>
__device__ __forceinline__ float wave_dot(const T* __restrict__ a, const T* __restrict__ b,
                                          int k, int lane) {
    float s = 0.f;
    for (int i = lane; i < k; i += 64) s += Elem<T>::load(a + i) * Elem<T>::load(b + i);
    return wave_sum_f32(s);
}

__device__ __forceinline__ float silu_ref(float a) { return a / (1.f + expf(-a)); }

template <typename T, bool GATED>
__global__ __launch_bounds__(256) void linear_simple_kernel(const T* __restrict__ x,
                                                            const T* __restrict__ w0,
                                                            const T* __restrict__ w1,
                                                            const T* residual, T* y, int64_t m,
                                                            int k_in, int n_out) {
    const int lane = threadIdx.x & 63;
    const int64_t o = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (o >= m * n_out) return;
    const int64_t row = o / n_out;
    const int f = (int)(o % n_out);
    const T* xr = x + row * k_in;
    const float a = wave_dot(xr, w0 + (int64_t)f * k_in, k_in, lane);
    float out;
    if (GATED) {
        const float b = wave_dot(xr, w1 + (int64_t)f * k_in, k_in, lane);
        const float ar = Elem<T>::to_f32(Elem<T>::from_f32(a));
        const float br = Elem<T>::to_f32(Elem<T>::from_f32(b));
        const float s = Elem<T>::to_f32(Elem<T>::from_f32(silu_ref(ar)));
        out = s * br;
    } else {
        out = a;
        if (residual) out = Elem<T>::to_f32(Elem<T>::from_f32(a)) + Elem<T>::load(residual + o);
    }
    if (lane == 0) y[o] = Elem<T>::from_f32(out);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <typename T>
pkv_status rmsnorm_typed(const void* h, const int32_t* row_idx, const void* weight, float eps,
                         void* y, int64_t m, int64_t hidden, hipStream_t st) {
    const unsigned blocks = (unsigned)ceil_div(m, 4);
    const bool in_regs = hidden * (int64_t)sizeof(T) <= 8 * 64 * 16;
    if (in_regs)
        hipLaunchKernelGGL((rmsnorm_rows_kernel<T, true>), dim3(blocks), dim3(256), 0, st,
                           (const T*)h, row_idx, (const T*)weight, eps, (T*)y, (int)m, (int)hidden);
    else
        hipLaunchKernelGGL((rmsnorm_rows_kernel<T, false>), dim3(blocks), dim3(256), 0, st,
                           (const T*)h, row_idx, (const T*)weight, eps, (T*)y, (int)m, (int)hidden);
    return launch_status();
}

template <typename T>
pkv_status linear_simple(bool gated, const void* x, const void* w0, const void* w1,
                         const void* residual, void* y, int64_t m, int64_t k_in, int64_t n_out,
                         hipStream_t st) {
    const int64_t blocks = ceil_div(m * n_out, 4);
    if (blocks > 0x7fffffff) return PKV_ERR_SHAPE;
    if (gated)
        hipLaunchKernelGGL((linear_simple_kernel<T, true>), dim3((unsigned)blocks), dim3(256), 0,
                           st, (const T*)x, (const T*)w0, (const T*)w1, (const T*)nullptr, (T*)y,
                           m, (int)k_in, (int)n_out);
    else
        hipLaunchKernelGGL((linear_simple_kernel<T, false>), dim3((unsigned)blocks), dim3(256), 0,
                           st, (const T*)x, (const T*)w0, (const T*)nullptr, (const T*)residual,
                           (T*)y, m, (int)k_in, (int)n_out);
    return launch_status();
}

}  // namespace

pkv_status launch_rmsnorm_rows(int dtype, const void* h, const int32_t* row_idx,
                               const void* weight, float eps, void* y, int64_t m,
                               int64_t hidden, hipStream_t st) {
    if (!aligned16(h) || !aligned16(weight) || !aligned16(y)) return PKV_ERR_UNSUPPORTED;
    return dtype == PKV_BF16
               ? rmsnorm_typed<bf16_t>(h, row_idx, weight, eps, y, m, hidden, st)
               : rmsnorm_typed<float>(h, row_idx, weight, eps, y, m, hidden, st);
}

pkv_status launch_gather_rows(int dtype, const void* src, const int32_t* row_idx, void* dst,
                              int64_t m, int64_t width, hipStream_t st) {
    if (!aligned16(src) || !aligned16(dst)) return PKV_ERR_UNSUPPORTED;
    const int chunks = (int)(width * (dtype == PKV_BF16 ? 2 : 4) / 16);
    const int64_t total = m * chunks;
    const int64_t blocks = ceil_div(total, 256);
    if (blocks > 0x7fffffff) return PKV_ERR_SHAPE;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       (const uint4*)src, row_idx, (uint4*)dst, total, chunks);
    return launch_status();
}

size_t glue_ws_bytes(int dtype, int64_t m, int64_t k_in, int64_t n_out) {
    if (dtype != PKV_BF16) return 0;
    if (!linear_dma_supported(kProjPlain, m, k_in, n_out) &&
        !linear_dma_supported(kProjGated, m, k_in, n_out))
        return 0;
    return linear_dma_partial_bytes(m);
}

pkv_status launch_linear_rows(int dtype, bool gated, const void* x, const void* w0,
                              const void* w1, const void* residual, void* y, int64_t m,
                              int64_t k_in, int64_t n_out, void* ws, hipStream_t st) {
    const int mode = gated ? kProjGated : kProjPlain;
    if (dtype == PKV_BF16 && linear_dma_supported(mode, m, k_in, n_out) && aligned16(x) &&
        aligned16(w0) && aligned16(y) && (!gated || aligned16(w1)) &&
        (!residual || aligned16(residual)))
        return launch_linear_dma(mode, (const bf16_t*)x, (const bf16_t*)w0, (const bf16_t*)w1,
                                 (const bf16_t*)residual, (bf16_t*)y, m, k_in, n_out, (float*)ws,
                                 st);
    return dtype == PKV_BF16
               ? linear_simple<bf16_t>(gated, x, w0, w1, residual, y, m, k_in, n_out, st)
               : linear_simple<float>(gated, x, w0, w1, residual, y, m, k_in, n_out, st);
}

}  // namespace pkv
