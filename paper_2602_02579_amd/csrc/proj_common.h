// Declarations shared by the MFMA projection kernels (gfx950, bf16).
#pragma once

#include "pkv_common.h"

namespace pkv {

struct ProjParams {
    const bf16_t* hidden;
    const int32_t* row_idx;
    const bf16_t* w[3];   // wq, wk, wv
    bf16_t* out[3];       // q_out, k_out, v_out (may be null)
    const float2* cs;     // [m, D/2] (cos, sin) of every output row's position
    int m, hid, hq, hkv;
    int tile_begin[4];    // first feature tile of Q, K, V, end
    float* partial;       // [n_ksplit, m, 256 * tile_begin[3]] fp32, used when n_ksplit > 1
    int n_ksplit;         // splits of the contraction (1 = none)
};

// head_dim 128, 256 x 256 output tiles, operands brought into LDS by direct
// global->LDS loads (gather_qkv_proj_dma.hip).  tile_begin counts tiles of
// 256 output features (two heads).
constexpr int kProjDmaTile = 256;
bool proj_dma128_supported(const pkv_layer_cfg& cfg, int64_t m);
// bytes of fp32 partials that a launch with m rows may need (0 when the launch is large
// enough to fill the chip without splitting the contraction)
size_t proj_dma128_partial_bytes(const pkv_layer_cfg& cfg, int64_t m);
pkv_status launch_proj_dma128(const ProjParams& p, hipStream_t st);

}  // namespace pkv
