// Shared device/host helpers of the pkv kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pkv.h"

namespace pkv {

// ---- storage element types -------------------------------------------------
// bf16 is kept as the compiler's native __bf16; fp32 <-> bf16 conversions go
// through the hardware convert (round to nearest even).
typedef __bf16 bf16_t;

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ float to_f32(float v) { return v; }
    static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p) { return (float)*p; }
    static __device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
    static __device__ __forceinline__ bf16_t from_f32(float v) { return (bf16_t)v; }
};

// 16-byte vector of storage elements (4 floats or 8 bf16)
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    typedef float type __attribute__((ext_vector_type(4)));
};
template <> struct Vec16<bf16_t> {
    static constexpr int N = 8;
    typedef bf16_t type __attribute__((ext_vector_type(8)));
};

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// ---- rotary frequency table, passed to kernels by value --------------------
// inv_freq[i] = theta^(-2i/D), computed on the host in double.
constexpr int kMaxHalfDim = 128;  // head_dim <= 256
struct RopeTable {
    double inv_freq[kMaxHalfDim];
};
void fill_rope_table(RopeTable* t, int head_dim, double theta);

// sin/cos of pos * inv_freq with the product and the reduction to
// [-pi, pi] done in double, so that positions in the hundreds of thousands
// lose nothing; the reduced angle goes through the fp32 sincos.
__device__ __forceinline__ void rope_sincos(double pos, double inv_freq,
                                            float* s, float* c) {
    const double two_pi = 6.283185307179586476925286766559;
    const double inv_two_pi = 0.15915494309189533576888376337251;
    double a = pos * inv_freq;
    double turns = rint(a * inv_two_pi);
    float r = (float)fma(-turns, two_pi, a);
    sincosf(r, s, c);
}

// ---- launch error mapping ---------------------------------------------------
inline pkv_status launch_status() {
    return hipGetLastError() == hipSuccess ? PKV_OK : PKV_ERR_LAUNCH;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- kernel launchers (one per source file) ---------------------------------
pkv_status launch_rope_restore(const pkv_layer_cfg& cfg, const void* k_in,
                               void* k_out, const int32_t* pos,
                               int64_t pos_base, int64_t n, hipStream_t st);

pkv_status launch_scatter_kv(const pkv_layer_cfg& cfg, const void* k_new,
                             const void* v_new, const int32_t* dst_row,
                             void* k_cache, void* v_cache, int64_t m,
                             hipStream_t st);

size_t topk_select_ws_bytes(int64_t n);
pkv_status launch_topk_select(const float* score, int64_t n, int64_t k,
                              int32_t* idx_out, void* ws, size_t ws_bytes, hipStream_t st);

size_t query_score_ws_bytes(const pkv_layer_cfg& cfg, int64_t n_ctx, int64_t nq);
pkv_status launch_query_score(const pkv_layer_cfg& cfg, const void* q,
                              const void* k, float* score, int64_t nq,
                              int64_t n_ctx, float scale, int accumulate,
                              void* ws, hipStream_t st);

pkv_status launch_query_score_lse(const pkv_layer_cfg& cfg, const void* q, const void* k,
                                  const float* lse, const int32_t* row_pos, float* score,
                                  int64_t nq, int64_t n_ctx, float scale, int accumulate,
                                  void* ws, hipStream_t st);

pkv_status launch_gather_qkv_proj(const pkv_layer_cfg& cfg, const void* hidden,
                                  const int32_t* row_idx, const int32_t* row_pos,
                                  const void* wq, const void* wk, const void* wv,
                                  const pkv_proj_variant* var, const int32_t* dst_row,
                                  void* q_out, void* k_out, void* v_out, int64_t m, void* ws,
                                  hipStream_t st);
size_t gather_qkv_proj_ws_bytes(const pkv_layer_cfg& cfg, int64_t m);

// ctx_keys > 0 with lse_ctx_out: also the log-sum-exp over the keys below ctx_keys
size_t sparse_row_attn_ws_bytes(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m,
                                int64_t ctx_keys = 0);
bool sparse_row_attn_ctx_lse_supported(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m,
                                       int64_t ctx_keys);
pkv_status launch_sparse_row_attn(const pkv_layer_cfg& cfg, const void* q,
                                  const void* k_cache, const void* v_cache,
                                  const int32_t* row_pos, void* out,
                                  float* lse_out, int64_t m, int64_t n_keys,
                                  float scale, void* ws, hipStream_t st,
                                  int64_t ctx_keys = 0, float* lse_ctx_out = nullptr);

// layer glue (layer_glue.hip); dtype is a pkv_dtype
pkv_status launch_rmsnorm_rows(int dtype, const void* h, const int32_t* row_idx,
                               const void* weight, float eps, void* y, int64_t m,
                               int64_t hidden, hipStream_t st);
pkv_status launch_gather_rows(int dtype, const void* src, const int32_t* row_idx, void* dst,
                              int64_t m, int64_t width, hipStream_t st);
size_t glue_ws_bytes(int dtype, int64_t m, int64_t k_in, int64_t n_out);
pkv_status launch_linear_rows(int dtype, bool gated, const void* x, const void* w0,
                              const void* w1, const void* residual, void* y, int64_t m,
                              int64_t k_in, int64_t n_out, void* ws, hipStream_t st);

}  // namespace pkv
