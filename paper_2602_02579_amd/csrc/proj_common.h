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
    // plain and gated launches only (launch_linear_dma): y = out[0] with rows of n_out
    // elements, w[0] (and w[1], the up matrix of the gated form); mat is always 0
    const bf16_t* residual;   // [m, n_out] or null
    int n_out;
    // Q | K | V launches of block variants: additive bias of each projection
    // ([heads * D] or null) and gains of the per-head RMS norm of Q and K applied before
    // the rotation ([D] or null)
    const bf16_t* bias[3];
    const bf16_t* norm_w[2];
    float norm_eps;
    // fused cache update: K and V of output row i go to row dst_row[i] of out[1] / out[2]
    // (the caches) instead of row i; null = plain outputs.  Q is never redirected.
    const int32_t* dst_row;
};

// what the tile's epilogue does with the accumulators
enum ProjMode {
    kProjRope = 0,    // Q | K | V heads, rotary pairs turned (the hot path)
    kProjPlain = 1,   // y = round(x W^T) (+ residual, rounded again)
    kProjGated = 2,   // y = round(round(silu(round(x Wg^T))) * round(x Wu^T))
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

// The same tile kernel as a plain or gated linear layer over m rows of k_in inputs.
// mode kProjPlain: n_out % 256 == 0; kProjGated: n_out % 128 == 0 (a tile then holds
// 2 x (64 gate rows + 64 up rows), so that a lane owns gate and up of one output).
bool linear_dma_supported(int mode, int64_t m, int64_t k_in, int64_t n_out);
size_t linear_dma_partial_bytes(int64_t m);
pkv_status launch_linear_dma(int mode, const bf16_t* x, const bf16_t* w0, const bf16_t* w1,
                             const bf16_t* residual, bf16_t* y, int64_t m, int64_t k_in,
                             int64_t n_out, float* partial, hipStream_t st);

}  // namespace pkv
