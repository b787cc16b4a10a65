// Declarations shared by the MFMA attention kernels (gfx950, bf16).
#pragma once

#include "pkv_common.h"

namespace pkv {

constexpr int kBN = 64;           // keys per LDS tile
constexpr int kAttnThreads = 256; // 4 waves per workgroup

struct AttnParams {
    const bf16_t* q;
    const bf16_t* k;
    const bf16_t* vt;        // [hkv, D, n_pad], zero beyond n_keys
    const bf16_t* v;         // [n_keys, hkv, D] as the cache holds it, or nullptr: when set, the
                             // eight-wave pipelined kernel and the exact kernel that redoes its
                             // marked tiles read it, and vt is not used
    const int32_t* row_pos;  // [m] or nullptr when fixed_limit >= 0
    bf16_t* out;             // [m, hq, D]
    float* lse;              // [m, hq] or nullptr
    float* part_ml;          // [n_splits, m*hq, 2] (max in raw logits, sum) or nullptr
    int* flags;              // [n_tiles, hkv]: written by the pipelined kernel (1 = redo the
                             // tile), read by the exact kernel when not nullptr
    int* queue;              // [hkv] next unclaimed row tile per kv head, zero before the
                             // launch (pipelined kernel only)
    float* part_o;           // [dma_splits, m, hq, D] normalised partial outputs, and
    float* part_lse;         // [dma_splits, m, hq] their log-sum-exp (pipelined kernel with
                             // dma_splits > 1 only)
    float* lse_ctx;          // [m, hq] or nullptr: log-sum-exp over the keys below ctx_keys
    int ctx_keys;            // a multiple of dma_split_len (and of 64) when lse_ctx is set
    int dma_splits, dma_split_len;   // key ranges per row tile in the pipelined kernel
    int m, n_keys, n_pad, hq, hkv, group, bm, n_tiles, n_splits, split_len;
    int fixed_limit;         // >= 0: every row sees keys 0..fixed_limit
    float scale_log2;        // softmax scale * log2(e)
    float scale;
};

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// head_dim 128 attention proper: software-pipelined, K / V^T tiles brought
// into LDS by direct global->LDS loads (sparse_row_attn_dma.hip)
pkv_status launch_attn_dma128(const AttnParams& p, hipStream_t st);
// its main kernel with eight waves of 32 columns per workgroup (sparse_row_attn_w8.hip)
pkv_status launch_attn_w8_main(const AttnParams& p, int n_cu, hipStream_t st);
// Where launch_attn_dma128's main kernel can take the values from: 1 = only from a V^T copy
// made by a pre-pass (the four-wave kernel, PKV_ATTN_WAVES=4, or PKV_ATTN_VT=1 in the
// environment), 0 = always from the cache as it is (PKV_ATTN_VT=0), -1 = either, the caller
// chooses by size.  The environment settings exist for comparisons and tests (PKV_ATTN_VT is
// read at every call, PKV_ATTN_WAVES once).
int attn_dma128_v_source();

}  // namespace pkv
