// Declarations shared by the query-score kernels (gfx950, bf16).
#pragma once

#include "pkv_common.h"

namespace pkv {

struct ScoreParams {
    const bf16_t* q;        // [nq, hq, D]
    const bf16_t* k;        // [n_ctx, hkv, D]
    float* part_ml;         // pass 1 out: [n_splits, nq * hq, 2] (max in raw logits, sum)
    const float* lse2;      // pass 2 in:  [nq * hq] normaliser, times lse_factor = its log2-domain
    float lse_factor;       //             value (1, or log2(e) for a natural-log normaliser)
    float* part_score;      // pass 2 out: [n_parts, n_ctx]
    int nq, n_ctx, hq, hkv, group;
    int n_cblk;             // blocks of 256 columns per kv group
    int n_splits, split_len;
    float scale_log2;
};

struct ScorePlan {
    int n_cblk, n_splits, split_len;
    int n_parts;            // partial scores per key: n_cblk * hkv * 4 waves
};

// head_dim 128: keys streamed through LDS by direct global->LDS loads
// (query_score_dma.hip)
bool score_dma128_supported(const pkv_layer_cfg& cfg, int64_t n_ctx, int64_t nq);
ScorePlan plan_score_dma128(const pkv_layer_cfg& cfg, int64_t n_ctx, int64_t nq);
pkv_status launch_score_dma128(int pass, const ScoreParams& p, hipStream_t st);

}  // namespace pkv
