// Step 4a on the matrix cores, head_dim 128, bf16: the gathered projection
// C^T[features, tokens] = W . X^T with the rotation of Q and K fused into the
// store.  (Paper: Algorithm 1, "Recompute KV cache at layer l" / "Calculate
// user query KV cache"; Appendix E: only the selected rows go through the
// projection.)
//
// One workgroup (4 waves, 2 x 2) owns 256 tokens x 256 output features (two
// heads); a wave owns 128 tokens x one head as 4 x 4 accumulators of
// v_mfma_f32_32x32x16_bf16 with the features on the accumulator rows.  A lane
// then holds, for one token, features 8j + 4(l/32) + {0..3} of every 32-block:
// both members (i, i + 64) of a rotary pair sit in the same lane and register
// index, and four consecutive features make one 8-byte piece of the output row.
//
// The contraction runs in steps of 32 through a 5-stage LDS ring filled by
// direct global->LDS loads (16 bytes per lane; the gather is free, every lane
// carries its own row pointer).  A row of a stage is 64 bytes; the 16-byte
// chunk c of row r is stored at position c ^ ((r >> 2) & 3), which makes both
// the 1 KB-contiguous fill and the ds_read_b128 of the MFMA operands
// conflict-free.  One barrier per stage, placed between the two 16-wide
// contraction sub-steps so that the operands of the next stage are already in
// flight while the second sub-step's MFMAs run.
//
// Tiles are numbered so that each XCD (workgroup id mod 8) works through its own
// contiguous run of tiles, 8 token tiles deep, and its L2 sees few distinct
// operand panels at a time.
//
// A launch with few rows (the user-query projection of the scoring stage: 128 rows,
// 16 tiles) cannot fill 256 CUs with tiles alone, so its contraction is split: every
// split writes fp32 partial tiles, and a second small kernel adds them in a fixed
// order, rotates and rounds (deterministic: no atomics).
#include <atomic>

#include "proj_common.h"

namespace pkv {

namespace {

constexpr int D = 128;
constexpr int T = kProjDmaTile;                  // tokens and features per tile
constexpr int BK = 32;                           // contraction per stage
constexpr int NS = 5;                            // LDS stages
constexpr int kRowBytes = BK * 2;                // 64
constexpr int kOperandBytes = T * kRowBytes;     // 16 KB: 256 rows of one operand
constexpr int kStageBytes = 2 * kOperandBytes;   // token rows, then feature rows
constexpr int kLdsBytes = NS * kStageBytes;      // 160 KB, all of a CU's LDS
constexpr int kEpiStride = 272;                  // bytes per token of the store staging
constexpr int kEpiStrideF32 = 528;               // same for fp32 partial tiles (32 tokens)
constexpr int kGroup = 8;                        // token tiles per group

// 16 bytes per lane from global memory straight into LDS: lane i of the wave
// writes LDS bytes [lds_base + 16 i, +16); lds_base must be wave-uniform.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, off"
        :
        : "s"(lds_base), "v"(gptr)
        : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// silu(a) = a / (1 + e^-a) with the hardware reciprocal (1 ulp): the result is rounded to
// bf16 right away, and a full-precision division would cost ten instructions per element
__device__ __forceinline__ float silu_f32(float a) {
    return a * __builtin_amdgcn_rcpf(1.f + __expf(-a));
}

// EXTRA (Q | K | V mode only): the launch has projection biases, per-head norm gains and/or
// a fused cache update (K/V rows stored at dst_row)
// what a tile is and which part of it a lane owns (filled by the kernels, read by the
// epilogue)
struct TileCtx {
    int lane, wave, hh, l32, wt, wf;
    int split, ft, mat, feat0, row0, heads_out;
    bf16_t* out;
};

// rotate pairs in registers / add the residual / gate, round, stage through LDS, store
// 16 B per lane; or store the fp32 partial tile of a split contraction.  Called after the
// main loop, when nothing is still writing the LDS stages.
template <int MODE, bool EXTRA>
__device__ __forceinline__ void tile_epilogue(const ProjParams& p, f32x16 (&acc)[4][4],
                                              const TileCtx& c, unsigned char* smem) {
    const int lane = c.lane, wave = c.wave, hh = c.hh, l32 = c.l32, wt = c.wt, wf = c.wf;
    const int split = c.split, ft = c.ft, mat = c.mat, feat0 = c.feat0, row0 = c.row0;
    const int heads_out = c.heads_out;
    bf16_t* out = c.out;
    // ---- epilogue: rotate pairs in registers, round once, stage, store 16 B per lane ----
    if (out == nullptr) return;   // uniform over the workgroup
    __syncthreads();              // LDS stages are free
    if (p.n_ksplit > 1) {
        // fp32 partial tile of this split, staged so that a lane stores 16 B and a
        // row 512 B: partial[split][row][256 ft + 128 wf + feature]
        unsigned char* epf = smem + wave * (32 * kEpiStrideF32);
        const int f_total = T * p.tile_begin[3];
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
            const int rbase = row0 + wt * 128 + tb * 32;
            if (rbase >= p.m) break;   // wave-uniform
            unsigned char* erow = epf + l32 * kEpiStrideF32;
#pragma unroll
            for (int fb = 0; fb < 4; ++fb)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[fb][tb][4 * j + e];
                    *reinterpret_cast<f32x4*>(erow + (fb * 32 + 8 * j + 4 * hh) * 4) = v;
                }
#pragma unroll
            for (int it = 0; it < 16; ++it) {
                const int idx = it * 64 + lane;
                const int tok = idx >> 5, ch = idx & 31;
                const int row = rbase + tok;
                const f32x4 v = *reinterpret_cast<const f32x4*>(epf + tok * kEpiStrideF32 + ch * 16);
                if (row < p.m)
                    *reinterpret_cast<f32x4*>(p.partial + ((int64_t)split * p.m + row) * f_total +
                                              ft * T + wf * 128 + ch * 4) = v;
            }
        }
        return;
    }
    unsigned char* epi = smem + wave * (64 * kEpiStride);
    if (MODE == kProjPlain) {
        // the wave's 128 tokens x 128 outputs: round the products, stage, then add the
        // residual (if any) 16 B per lane and round again
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int tbl = 0; tbl < 2; ++tbl) {
                const int tb = half * 2 + tbl;
                unsigned char* erow = epi + (tbl * 32 + l32) * kEpiStride;
#pragma unroll
                for (int fb = 0; fb < 4; ++fb)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        bf16x4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = (bf16_t)acc[fb][tb][4 * j + e];
                        *reinterpret_cast<bf16x4*>(erow + (fb * 32 + 8 * j + 4 * hh) * 2) = v;
                    }
            }
#pragma unroll
            for (int it = 0; it < 16; ++it) {
                const int idx = it * 64 + lane;
                const int tok = idx >> 4, ch = idx & 15;
                const int row = row0 + wt * 128 + half * 64 + tok;
                bf16x8 v = *reinterpret_cast<const bf16x8*>(epi + tok * kEpiStride + ch * 16);
                if (row < p.m) {
                    const int64_t o = (int64_t)row * p.n_out + feat0 + wf * 128 + ch * 8;
                    if (p.residual) {
                        const bf16x8 r = *reinterpret_cast<const bf16x8*>(p.residual + o);
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = (bf16_t)((float)v[e] + (float)r[e]);
                    }
                    *reinterpret_cast<bf16x8*>(out + o) = v;
                }
            }
        }
        return;
    }
    if (MODE == kProjGated) {
        // the wave's 128 tokens x 64 outputs: gate in blocks 0, 1 and up in blocks 2, 3
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int tbl = 0; tbl < 2; ++tbl) {
                const int tb = half * 2 + tbl;
                unsigned char* erow = epi + (tbl * 32 + l32) * kEpiStride;
#pragma unroll
                for (int fbp = 0; fbp < 2; ++fbp)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        bf16x4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float a = (float)(bf16_t)acc[fbp][tb][4 * j + e];
                            const float b = (float)(bf16_t)acc[fbp + 2][tb][4 * j + e];
                            const float s = (float)(bf16_t)silu_f32(a);
                            v[e] = (bf16_t)(s * b);
                        }
                        *reinterpret_cast<bf16x4*>(erow + (fbp * 32 + 8 * j + 4 * hh) * 2) = v;
                    }
            }
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int idx = it * 64 + lane;
                const int tok = idx >> 3, ch = idx & 7;
                const int row = row0 + wt * 128 + half * 64 + tok;
                const uint4 v = *reinterpret_cast<const uint4*>(epi + tok * kEpiStride + ch * 16);
                if (row < p.m)
                    *reinterpret_cast<uint4*>(out + (int64_t)row * p.n_out + ft * 128 + wf * 64 +
                                              ch * 8) = v;
            }
        }
        return;
    }
    const int head = feat0 / D + wf;
    const bool rotate = mat != 2;
    // block variants: bias of this head's features, gains of the head norm (Q and K only)
    const bf16_t* bias = EXTRA && p.bias[mat] ? p.bias[mat] + head * D : nullptr;
    const bf16_t* gain = EXTRA && mat != 2 ? p.norm_w[mat] : nullptr;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int tbl = 0; tbl < 2; ++tbl) {
            const int tb = half * 2 + tbl;
            const int row = min(row0 + wt * 128 + tb * 32 + l32, p.m - 1);
            const float4* cs = reinterpret_cast<const float4*>(p.cs + (int64_t)row * (D / 2));
            unsigned char* erow = epi + (tbl * 32 + l32) * kEpiStride;
            float rnorm = 1.f;
            if (EXTRA) {
                if (bias) {
#pragma unroll
                    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const bf16x4 bv =
                                *reinterpret_cast<const bf16x4*>(bias + fb * 32 + 8 * j + 4 * hh);
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[fb][tb][4 * j + e] += (float)bv[e];
                        }
                }
                if (gain) {
                    // the lane holds 64 of the token's 128 features, lane ^ 32 the other 64
                    float ss = 0.f;
#pragma unroll
                    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) ss += acc[fb][tb][r] * acc[fb][tb][r];
                    ss += __shfl_xor(ss, 32);
                    rnorm = 1.0f / sqrtf(ss * (1.0f / D) + p.norm_eps);
                }
            }
#pragma unroll
            for (int fbp = 0; fbp < 2; ++fbp)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i0 = fbp * 32 + 8 * j + 4 * hh;   // pair index of element 0
                    float a[4], b[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        a[e] = acc[fbp][tb][4 * j + e];
                        b[e] = acc[fbp + 2][tb][4 * j + e];
                    }
                    if (EXTRA && gain) {
                        const bf16x4 ga = *reinterpret_cast<const bf16x4*>(gain + i0);
                        const bf16x4 gb = *reinterpret_cast<const bf16x4*>(gain + i0 + D / 2);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            a[e] = a[e] * rnorm * (float)ga[e];
                            b[e] = b[e] * rnorm * (float)gb[e];
                        }
                    }
                    if (rotate) {
                        const float4 t0 = cs[i0 / 2], t1 = cs[i0 / 2 + 1];
                        const float c[4] = {t0.x, t0.z, t1.x, t1.z};
                        const float s[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float ra = a[e] * c[e] - b[e] * s[e];
                            const float rb = b[e] * c[e] + a[e] * s[e];
                            a[e] = ra;
                            b[e] = rb;
                        }
                    }
                    bf16x4 va, vb;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        va[e] = (bf16_t)a[e];
                        vb[e] = (bf16_t)b[e];
                    }
                    *reinterpret_cast<bf16x4*>(erow + i0 * 2) = va;
                    *reinterpret_cast<bf16x4*>(erow + (i0 + D / 2) * 2) = vb;
                }
        }
        // the wave's own 64 tokens x 256 B, now 16 B per lane and 256 B per row
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int idx = it * 64 + lane;
            const int tok = idx >> 4, ch = idx & 15;
            const int row = row0 + wt * 128 + half * 64 + tok;
            const uint4 v = *reinterpret_cast<const uint4*>(epi + tok * kEpiStride + ch * 16);
            if (row < p.m) {
                const int64_t orow = (EXTRA && mat != 0 && p.dst_row) ? p.dst_row[row] : row;
                *reinterpret_cast<uint4*>(out + (orow * heads_out + head) * D + ch * 8) = v;
            }
        }
    }
}


template <int MODE, bool EXTRA = false>
__global__ __launch_bounds__(256) void proj_dma_kernel(ProjParams p, int n_tok_tiles,
                                                       int n_tiles, int per_xcd) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5, l32 = lane & 31;
    const int wt = wave >> 1, wf = wave & 1;

    // ---- which tile --------------------------------------------------------------
    int logical = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (logical >= n_tiles * p.n_ksplit) return;
    const int split = logical / n_tiles;
    logical -= split * n_tiles;
    const int n_feat_tiles = p.tile_begin[3];
    const int per_group = kGroup * n_feat_tiles;
    const int group = logical / per_group;
    const int first_tok = group * kGroup;
    const int rows_in_group = min(kGroup, n_tok_tiles - first_tok);
    const int within = logical - group * per_group;
    const int tok_tile = first_tok + within % rows_in_group;
    const int ft = within / rows_in_group;
    int mat = 0;
    if (MODE == kProjRope) {
        if (ft >= p.tile_begin[1]) mat = 1;
        if (ft >= p.tile_begin[2]) mat = 2;
    }
    const int feat0 = (ft - p.tile_begin[mat]) * T;   // first output feature of the tile
    const bf16_t* w = p.w[mat];
    bf16_t* out = p.out[mat];
    const int heads_out = mat == 0 ? p.hq : p.hkv;
    const int row0 = tok_tile * T;

    const int n_k = p.hid / BK / p.n_ksplit;   // stages of this split; >= NS (launcher)
    const int k_begin = split * n_k * BK;

    // ---- fill side: wave w, instruction j covers rows 16 (4w + j) .. + 16 ------------
    const int sw = (lane & 3) ^ ((lane >> 4) & 3);   // global chunk that lands at lane & 3
    const bf16_t* xptr[4];
    const bf16_t* wptr[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = (wave * 4 + j) * 16 + (lane >> 2);
        const int gr = min(row0 + r, p.m - 1);
        const int64_t src_row = p.row_idx ? p.row_idx[gr] : gr;
        xptr[j] = p.hidden + src_row * p.hid + k_begin + sw * 8;
        if (MODE == kProjGated) {
            // tile row r: half r / 128 of the tile's 128 outputs, then 64 gate rows and
            // 64 up rows, so that accumulator blocks (0, 1) and (2, 3) of a wave hold
            // gate and up of the same outputs
            const int f = ft * 128 + (r >> 7) * 64 + (r & 63);
            wptr[j] = p.w[(r >> 6) & 1] + (int64_t)f * p.hid + k_begin + sw * 8;
        } else {
            wptr[j] = w + (int64_t)(feat0 + r) * p.hid + k_begin + sw * 8;
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const uint32_t lds_fill = __builtin_amdgcn_readfirstlane(lds0 + wave * 4 * 1024);
    // one fill instruction: 16 rows of the token operand (which = 0) or of the
    // feature operand (which = 1).  adv is BK, or 0 once the last stage has been
    // requested: the ring then keeps re-reading that stage into slots nobody reads
    // any more, which keeps the loop and its wait counts uniform.
    auto issue_one = [&](int stage, int j, int which, int adv) {
        const uint32_t base = lds_fill + stage * kStageBytes + j * 1024;
        if (which == 0) {
            dma16(xptr[j], base);
            xptr[j] += adv;
        } else {
            dma16(wptr[j], base + kOperandBytes);
            wptr[j] += adv;
        }
    };

    // ---- read side -----------------------------------------------------------------
    // operand of row r, sub-step ks: chunk ks*2 + hh at position chunk ^ ((r >> 2) & 3)
    int off_x[2], off_w[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int pos = (ks * 2 + hh) ^ ((l32 >> 2) & 3);
        off_x[ks] = (wt * 128 + l32) * kRowBytes + pos * 16;
        off_w[ks] = kOperandBytes + (wf * 128 + l32) * kRowBytes + pos * 16;
    }
    bf16x8 fx[2][4], fw[2][4];
    auto load_frags = [&](int stage, int ks, int slot) {
        const unsigned char* sb = smem + stage * kStageBytes;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            fw[slot][b] = *reinterpret_cast<const bf16x8*>(sb + off_w[ks] + b * 32 * kRowBytes);
            fx[slot][b] = *reinterpret_cast<const bf16x8*>(sb + off_x[ks] + b * 32 * kRowBytes);
        }
    };

    f32x16 acc[4][4];   // [feature block][token block]
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fb][tb][r] = 0.f;
    // 16 MFMAs of one contraction sub-step.  One fill instruction goes out after every
    // fourth MFMA (half a stage per sub-step), so the memory pipeline sees a steady
    // trickle instead of a burst that stalls the wave; the operands of the next
    // sub-step (stage lstage, sub-step lks) are read from LDS in the same rhythm,
    // two per four MFMAs, into the other register slot
    auto mfma16 = [&](int slot, int fill_stage, int j0, int adv, int lstage, int lks) {
        const unsigned char* sb = smem + lstage * kStageBytes;
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
            fw[slot ^ 1][fb] = *reinterpret_cast<const bf16x8*>(sb + off_w[lks] + fb * 32 * kRowBytes);
            fx[slot ^ 1][fb] = *reinterpret_cast<const bf16x8*>(sb + off_x[lks] + fb * 32 * kRowBytes);
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
                acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[slot][fb], fx[slot][tb],
                                                                      acc[fb][tb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            issue_one(fill_stage, j0 + (fb >> 1), fb & 1, adv);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // prologue: stages 0 .. NS-3 and the first half of stage NS-2 in flight
#pragma unroll
    for (int s = 0; s < NS - 2; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            issue_one(s, j, 0, BK);
            issue_one(s, j, 1, BK);
        }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        issue_one(NS - 2, j, 0, BK);
        issue_one(NS - 2, j, 1, BK);
    }
    wait_vm<8 * (NS - 3) + 4>();  // stage 0 of this wave has landed
    __syncthreads();              // ... and everyone's
    load_frags(0, 0, 0);
    int st_cur = 0;               // t mod NS
    for (int t = 0; t < n_k; ++t) {
        const int st_next = st_cur + 1 == NS ? 0 : st_cur + 1;
        const int st_fill = st_cur == 0 ? NS - 1 : st_cur - 1;          // (t + NS - 1) mod NS
        const int st_fill_b = st_fill == 0 ? NS - 1 : st_fill - 1;      // (t + NS - 2) mod NS
        mfma16(0, st_fill_b, 2, t + NS - 1 < n_k ? BK : 0, st_cur, 1);
        wait_vm<8 * (NS - 3)>();  // stage t+1 has landed; the younger ones stay in flight
        __syncthreads();          // ... for everyone; and everyone is done with stage t-1
        mfma16(1, st_fill, 0, t + NS < n_k ? BK : 0, st_next, 0);
        st_cur = st_next;
    }
    wait_vm<0>();                 // the ring's trailing fills must not land in the staging

    // ---- epilogue -----------------------------------------------------------------------
    TileCtx ctx;
    ctx.lane = lane; ctx.wave = wave; ctx.hh = hh; ctx.l32 = l32; ctx.wt = wt; ctx.wf = wf;
    ctx.split = split; ctx.ft = ft; ctx.mat = mat; ctx.feat0 = feat0; ctx.row0 = row0;
    ctx.heads_out = heads_out; ctx.out = out;
    tile_epilogue<MODE, EXTRA>(p, acc, ctx, smem);
}

// ---------------------------------------------------------------------------------------
// The same tile with the contraction in steps of 64 ("slabs"): every fill instruction
// fetches whole 128-byte lines (8 rows x 128 B), which the memory pipeline serves at
// 1.7 x the rate of the 64-byte row pieces of the kernel above and at a higher clock.
//
// LDS: a ring of 16 units of 8 KB; a unit is 64 rows x 128 B of one operand.  A step T
// needs four feature units W0..W3 (tile rows 64 i ..) and four token units X0..X3, where
// X_q holds the rows both token halves consume in quarter q of the step: tile rows
// 32 q .. + 32 and 128 + 32 q .. + 32.  Units of step T sit in slots 8 (T & 1) + (0..7).
// The 16-byte chunk c of unit row r is stored at position c ^ ((r >> 1) & 7): two 128-byte
// rows span the 64 banks, so the sixteen lanes that an operand read serves per clock (rows
// r .. r + 15, one logical chunk) must differ in (r & 1, position) - with c ^ (r & 7) rows r
// and r + 8 met in one bank group and every read took two passes (SQ_LDS_BANK_CONFLICT).
//
// A step is 64 MFMAs per wave in four quarters; quarter q multiplies the wave's four
// feature blocks by its token block q for all four 16-wide sub-steps.  The feature
// operands of a whole step live in registers (loaded during the second half of the
// previous step), so the W units of step T are free again when T begins and are refilled
// with step T + 2 during its first two quarters; X_q is free after quarter q - 1 and is
// refilled in quarters 2 and 3.  One barrier per quarter, two fill instructions per wave
// and unit, one fill instruction every four MFMAs, as in the kernel above.
// Needs an even number (>= 2) of steps per split.
constexpr int kUnitBytes = 64 * 128;
constexpr int kSlabLdsBytes = 16 * kUnitBytes;

template <int MODE, bool EXTRA = false>
__global__ __launch_bounds__(256) void proj_slab_kernel(ProjParams p, int n_tok_tiles,
                                                        int n_tiles, int per_xcd) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5, l32 = lane & 31;
    const int wt = wave >> 1, wf = wave & 1;

    // ---- which tile (as above) ---------------------------------------------------------
    int logical = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (logical >= n_tiles * p.n_ksplit) return;
    const int split = logical / n_tiles;
    logical -= split * n_tiles;
    const int n_feat_tiles = p.tile_begin[3];
    const int per_group = kGroup * n_feat_tiles;
    const int group = logical / per_group;
    const int first_tok = group * kGroup;
    const int rows_in_group = min(kGroup, n_tok_tiles - first_tok);
    const int within = logical - group * per_group;
    const int tok_tile = first_tok + within % rows_in_group;
    const int ft = within / rows_in_group;
    int mat = 0;
    if (MODE == kProjRope) {
        if (ft >= p.tile_begin[1]) mat = 1;
        if (ft >= p.tile_begin[2]) mat = 2;
    }
    const int feat0 = (ft - p.tile_begin[mat]) * T;
    const bf16_t* w = p.w[mat];
    bf16_t* out = p.out[mat];
    const int heads_out = mat == 0 ? p.hq : p.hkv;
    const int row0 = tok_tile * T;

    const int n_T = p.hid / 64 / p.n_ksplit;   // steps of this split: even, >= 2 (launcher)
    const int k_begin = split * n_T * 64;

    // ---- fill side: wave w issues instructions j = 0, 1 of every unit: unit rows
    // 8 (2 w + j) .. + 8; lane = (row in the eight, position), fetching the chunk that
    // belongs at that position: pos ^ ((unit row >> 1) & 7) = pos ^ (4 j + (row >> 1))
    const int rl = lane >> 3;
    const bf16_t* wptr[4][2];
    const bf16_t* xptr[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int ur = 8 * (2 * wave + j) + rl;   // row inside the unit
            const int gchunk = (lane & 7) ^ ((ur >> 1) & 7);
            const int r = 64 * i + ur;                // feature row of the tile
            if (MODE == kProjGated) {
                const int f = ft * 128 + (r >> 7) * 64 + (r & 63);
                wptr[i][j] = p.w[(r >> 6) & 1] + (int64_t)f * p.hid + k_begin + gchunk * 8;
            } else {
                wptr[i][j] = w + (int64_t)(feat0 + r) * p.hid + k_begin + gchunk * 8;
            }
            const int xr = ur < 32 ? 32 * i + ur : 96 + 32 * i + ur;   // token row of the tile
            const int gr = min(row0 + xr, p.m - 1);
            const int64_t src_row = p.row_idx ? p.row_idx[gr] : gr;
            xptr[i][j] = p.hidden + src_row * p.hid + k_begin + gchunk * 8;
        }
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const uint32_t lds_fill = __builtin_amdgcn_readfirstlane(lds0 + wave * 2 * 1024);
    // unit i of the feature (which = 1) or token (which = 0) operand of a step with
    // parity par; adv is 64, or 0 once the last step has been requested
    auto issue_w = [&](int par, int i, int j, int adv) {
        dma16(wptr[i][j], lds_fill + (par * 8 + i) * kUnitBytes + j * 1024);
        wptr[i][j] += adv;
    };
    auto issue_x = [&](int par, int i, int j, int adv) {
        dma16(xptr[i][j], lds_fill + (par * 8 + 4 + i) * kUnitBytes + j * 1024);
        xptr[i][j] += adv;
    };

    // ---- read side: byte offsets of the lane's operand pieces --------------------------
    // feature block fb: base_w + fb * 4096; token quarter q: base_x + q * 8192
    uint32_t base_w[2][4], base_x[2][4];
#pragma unroll
    for (int par = 0; par < 2; ++par)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const uint32_t swz = (uint32_t)(((2 * ks + hh) ^ ((l32 >> 1) & 7)) * 16);
            base_w[par][ks] = par * 8 * kUnitBytes + 2 * wf * kUnitBytes + l32 * 128 + swz;
            base_x[par][ks] = par * 8 * kUnitBytes + 4 * kUnitBytes + (wt * 32 + l32) * 128 + swz;
        }
    auto ld = [&](uint32_t off) { return *reinterpret_cast<const bf16x8*>(smem + off); };

    bf16x8 fw01[2][4][2];   // [step parity][feature block][sub-step 0, 1]
    bf16x8 fw23[4][2];      // [feature block][sub-step 2, 3]
    bf16x8 fx[2][4];        // [quarter parity][sub-step]

    f32x16 acc[4][4];   // [feature block][token block]
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fb][tb][r] = 0.f;

    // ---- prologue: steps 0 and 1 requested; operands of step 0, quarter 0 loaded --------
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int adv = par + 1 < n_T ? 64 : 0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) issue_w(par, i, j, adv);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) issue_x(par, i, j, adv);
    }
    wait_vm<22>();     // W0..W3 and X0 of step 0 (the first ten of 32 instructions) landed
    __syncthreads();
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
        fw01[0][fb][0] = ld(base_w[0][0] + fb * 4096);
        fw01[0][fb][1] = ld(base_w[0][1] + fb * 4096);
        fw23[fb][0] = ld(base_w[0][2] + fb * 4096);
        fw23[fb][1] = ld(base_w[0][3] + fb * 4096);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) fx[0][ks] = ld(base_x[0][ks]);
    __syncthreads();   // everybody holds step 0's feature operands: its W units may be refilled

    // One quarter: 16 MFMAs in four groups (sub-step outer, feature block inner) on token
    // block Q with the token operands fx[Q & 1]; one fill instruction after every group.
    // The LDS reads of the quarter (token operands of the next quarter; in quarter 2 the
    // sub-step 0, 1 feature operands of the next step into the other register set; in
    // quarter 3 the sub-step 2, 3 ones, each right after its last use - which is why
    // quarter 3 runs sub-steps 2, 3 first) all go out in the first three groups, so that
    // they have returned when the barrier that ends the quarter waits for them.
    // PAR = parity of the step.
#define PKV_QUARTER(PAR, Q, ADV)                                                          \
    {                                                                                     \
        _Pragma("unroll") for (int g_ = 0; g_ < 4; ++g_) {                                \
            const int ks = (Q) == 3 ? (g_ + 2) & 3 : g_;                                  \
            _Pragma("unroll") for (int fb = 0; fb < 4; ++fb) {                            \
                const bf16x8 a_ = ks < 2 ? fw01[PAR][fb][ks] : fw23[fb][ks - 2];          \
                acc[fb][Q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_, fx[(Q) & 1][ks], \
                                                                     acc[fb][Q], 0, 0, 0); \
                if ((Q) == 3 && ks >= 2)   /* last use: take step T + 1's operand */      \
                    fw23[fb][ks - 2] = ld(base_w[(PAR) ^ 1][ks] + fb * 4096);             \
            }                                                                             \
            __builtin_amdgcn_sched_barrier(0);                                            \
            /* fill: quarters 0, 1 -> feature units 2 Q, 2 Q + 1; 2, 3 -> token units */  \
            if ((Q) < 2) issue_w(PAR, 2 * (Q) + (g_ >> 1), g_ & 1, ADV);                  \
            else issue_x(PAR, 2 * ((Q) - 2) + (g_ >> 1), g_ & 1, ADV);                    \
            /* token operands of the next quarter: 2, 1, 1, 0 per group */                \
            _Pragma("unroll") for (int n_ = 0; n_ < 4; ++n_) {                            \
                if ((n_ < 2 ? 0 : n_ - 1) != g_) continue;                                \
                if ((Q) < 3) fx[((Q) + 1) & 1][n_] = ld(base_x[PAR][n_] + ((Q) + 1) * 8192); \
                else fx[0][n_] = ld(base_x[(PAR) ^ 1][n_]);                               \
            }                                                                             \
            /* quarter 2: feature operands of sub-steps 0, 1 of the next step: blocks     \
               0 | 1, 2 | 3 | - per group */                                              \
            if ((Q) == 2) {                                                               \
                _Pragma("unroll") for (int fb = 0; fb < 4; ++fb) {                        \
                    if ((fb == 0 ? 0 : fb == 3 ? 2 : 1) != g_) continue;                  \
                    fw01[(PAR) ^ 1][fb][0] = ld(base_w[(PAR) ^ 1][0] + fb * 4096);        \
                    fw01[(PAR) ^ 1][fb][1] = ld(base_w[(PAR) ^ 1][1] + fb * 4096);        \
                }                                                                         \
            }                                                                             \
            __builtin_amdgcn_sched_barrier(0);                                            \
        }                                                                                 \
    }
    // outstanding fills allowed at the barrier that ends quarter 0, 1, 2, 3 (see above):
    // what the next quarter reads was requested at least 22 / 16 / 18 / 20 instructions ago
#define PKV_STEP(PAR, ADV)                                                                \
    PKV_QUARTER(PAR, 0, ADV) wait_vm<22>(); __syncthreads();                              \
    PKV_QUARTER(PAR, 1, ADV) wait_vm<16>(); __syncthreads();                              \
    PKV_QUARTER(PAR, 2, ADV) wait_vm<18>(); __syncthreads();                              \
    PKV_QUARTER(PAR, 3, ADV) wait_vm<20>(); __syncthreads();

    for (int t = 0; t < n_T; t += 2) {
        const int adv0 = t + 3 < n_T ? 64 : 0;   // step t fetches step t + 2
        const int adv1 = t + 4 < n_T ? 64 : 0;
        PKV_STEP(0, adv0)
        PKV_STEP(1, adv1)
    }
#undef PKV_STEP
#undef PKV_QUARTER
    wait_vm<0>();                 // the ring's trailing fills must not land in the staging

    TileCtx ctx;
    ctx.lane = lane; ctx.wave = wave; ctx.hh = hh; ctx.l32 = l32; ctx.wt = wt; ctx.wf = wf;
    ctx.split = split; ctx.ft = ft; ctx.mat = mat; ctx.feat0 = feat0; ctx.row0 = row0;
    ctx.heads_out = heads_out; ctx.out = out;
    tile_epilogue<MODE, EXTRA>(p, acc, ctx, smem);
}

// adds the splits of the contraction in a fixed order, rotates, rounds once, stores.
// One thread per (row, head slot, pair index i): elements i and i + 64 of the head.
__global__ __launch_bounds__(256) void proj_splitk_finish_kernel(ProjParams p) {
    const int f_total = T * p.tile_begin[3];
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)p.m * (f_total / 2);
    if (idx >= total) return;
    const int i = (int)(idx % (D / 2));
    const int hs = (int)((idx / (D / 2)) % (f_total / D));   // head slot over Q | K | V
    const int row = (int)(idx / ((int64_t)(D / 2) * (f_total / D)));
    const int ft = hs / 2;
    int mat = 0;
    if (ft >= p.tile_begin[1]) mat = 1;
    if (ft >= p.tile_begin[2]) mat = 2;
    bf16_t* out = p.out[mat];
    if (out == nullptr) return;
    const int head = (ft - p.tile_begin[mat]) * 2 + (hs & 1);
    const int heads_out = mat == 0 ? p.hq : p.hkv;
    float a = 0.f, b = 0.f;
    for (int s = 0; s < p.n_ksplit; ++s) {
        const float* src = p.partial + ((int64_t)s * p.m + row) * f_total + hs * D + i;
        a += src[0];
        b += src[D / 2];
    }
    if (p.bias[mat]) {
        a += (float)p.bias[mat][head * D + i];
        b += (float)p.bias[mat][head * D + i + D / 2];
    }
    if (mat != 2 && p.norm_w[mat]) {
        // a wave is exactly one (row, head): its 64 lanes hold the head's 128 features
        float ss = a * a + b * b;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
        const float r = 1.0f / sqrtf(ss * (1.0f / D) + p.norm_eps);
        a = a * r * (float)p.norm_w[mat][i];
        b = b * r * (float)p.norm_w[mat][i + D / 2];
    }
    if (mat != 2) {
        const float2 t = p.cs[(int64_t)row * (D / 2) + i];
        const float ra = a * t.x - b * t.y;
        const float rb = b * t.x + a * t.y;
        a = ra;
        b = rb;
    }
    const int64_t orow = (mat != 0 && p.dst_row) ? p.dst_row[row] : row;
    bf16_t* o = out + (orow * heads_out + head) * D + i;
    o[0] = (bf16_t)a;
    o[D / 2] = (bf16_t)b;
}

// the same for the plain and the gated linear layers: one thread per (row, 4 outputs)
template <int MODE>
__global__ __launch_bounds__(256) void linear_splitk_finish_kernel(ProjParams p) {
    const int f_total = T * p.tile_begin[3];
    const int quads = p.n_out / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)p.m * quads) return;
    const int row = (int)(idx / quads);
    const int f = (int)(idx % quads) * 4;
    // column of output f in the tile order of the partials
    const int col = MODE == kProjGated ? (f >> 7) * T + ((f >> 6) & 1) * 128 + (f & 63) : f;
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < p.n_ksplit; ++s) {
        const float* src = p.partial + ((int64_t)s * p.m + row) * f_total + col;
        a += *reinterpret_cast<const f32x4*>(src);
        if (MODE == kProjGated) b += *reinterpret_cast<const f32x4*>(src + 64);
    }
    const int64_t o = (int64_t)row * p.n_out + f;
    bf16x4 v;
    if (MODE == kProjGated) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float ar = (float)(bf16_t)a[e], br = (float)(bf16_t)b[e];
            v[e] = (bf16_t)((float)(bf16_t)silu_f32(ar) * br);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16_t)a[e];
        if (p.residual) {
            const bf16x4 r = *reinterpret_cast<const bf16x4*>(p.residual + o);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (bf16_t)((float)v[e] + (float)r[e]);
        }
    }
    *reinterpret_cast<bf16x4*>(p.out[0] + o) = v;
}

// splits of the contraction for a launch of n_tiles tiles over n_k stages: the largest
// power of two that keeps the launch within ~256 workgroups and a split >= NS stages
int plan_ksplit(int64_t n_tiles, int n_k) {
    int ks = 1;
    while (ks < 16 && n_tiles * (ks * 2) <= 256 && n_k % (ks * 2) == 0 && n_k / (ks * 2) >= NS)
        ks *= 2;
    return ks;
}

}  // namespace

size_t proj_dma128_partial_bytes(const pkv_layer_cfg& cfg, int64_t m) {
    // n_ksplit * (features of the launch) <= 256 * 256 / (token tiles): see plan_ksplit
    const int64_t n_tok_tiles = ceil_div(m, T);
    if (n_tok_tiles > 128) return 0;
    (void)cfg;
    return (size_t)m * (size_t)(T * 256 / n_tok_tiles) * sizeof(float);
}

bool proj_dma128_supported(const pkv_layer_cfg& cfg, int64_t m) {
    return cfg.dtype == PKV_BF16 && cfg.head_dim == D && cfg.hidden % BK == 0 &&
           cfg.hidden / BK >= NS && cfg.n_q_heads % 2 == 0 && cfg.n_kv_heads % 2 == 0 &&
           m > 0 && m < (1 << 30);
}

namespace {

template <int MODE, bool EXTRA = false>
pkv_status launch_tiles(const ProjParams& p, hipStream_t st) {
    static std::atomic<bool> configured{false};   // set twice at worst: the calls are idempotent
    if (!configured.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(proj_dma_kernel<MODE, EXTRA>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(proj_slab_kernel<MODE, EXTRA>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kSlabLdsBytes) != hipSuccess)
            return PKV_ERR_LAUNCH;
        configured.store(true, std::memory_order_release);
    }
    const int n_tok_tiles = (int)ceil_div(p.m, T);
    const int64_t n_tiles = (int64_t)n_tok_tiles * p.tile_begin[3];
    if (n_tiles == 0) return PKV_OK;
    if (n_tiles > (1 << 30)) return PKV_ERR_SHAPE;
    ProjParams q = p;
    q.n_ksplit = plan_ksplit(n_tiles, p.hid / BK);
    if (q.n_ksplit > 1 && q.partial == nullptr) return PKV_ERR_WORKSPACE;
    const int per_xcd = (int)ceil_div(n_tiles * q.n_ksplit, 8);
    // contraction in slabs of 64 when every split has an even number of them
    if (p.hid % (128 * q.n_ksplit) == 0)
        hipLaunchKernelGGL((proj_slab_kernel<MODE, EXTRA>), dim3((unsigned)(per_xcd * 8)),
                           dim3(256), kSlabLdsBytes, st, q, n_tok_tiles, (int)n_tiles, per_xcd);
    else
        hipLaunchKernelGGL((proj_dma_kernel<MODE, EXTRA>), dim3((unsigned)(per_xcd * 8)),
                           dim3(256), kLdsBytes, st, q, n_tok_tiles, (int)n_tiles, per_xcd);
    if (q.n_ksplit > 1) {
        if (MODE == kProjRope) {
            const int64_t total = (int64_t)p.m * (T * p.tile_begin[3] / 2);
            hipLaunchKernelGGL(proj_splitk_finish_kernel, dim3((unsigned)ceil_div(total, 256)),
                               dim3(256), 0, st, q);
        } else {
            const int64_t total = (int64_t)p.m * (p.n_out / 4);
            hipLaunchKernelGGL(linear_splitk_finish_kernel<MODE>,
                               dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, st, q);
        }
    }
    return launch_status();
}

}  // namespace

pkv_status launch_proj_dma128(const ProjParams& p, hipStream_t st) {
    const bool extra = p.bias[0] || p.bias[1] || p.bias[2] || p.norm_w[0] || p.norm_w[1] ||
                       p.dst_row;
    return extra ? launch_tiles<kProjRope, true>(p, st) : launch_tiles<kProjRope, false>(p, st);
}

bool linear_dma_supported(int mode, int64_t m, int64_t k_in, int64_t n_out) {
    const int64_t per_tile = mode == kProjGated ? T / 2 : T;
    return m > 0 && m < (1 << 30) && k_in % BK == 0 && k_in / BK >= NS && k_in < (1 << 30) &&
           n_out > 0 && n_out % per_tile == 0 && n_out < (1 << 30);
}

size_t linear_dma_partial_bytes(int64_t m) {
    // as for the Q/K/V launch: splits x features <= 256 tiles' worth
    const int64_t n_tok_tiles = ceil_div(m, T);
    if (m <= 0 || n_tok_tiles > 128) return 0;
    return (size_t)m * (size_t)(T * 256 / n_tok_tiles) * sizeof(float);
}

pkv_status launch_linear_dma(int mode, const bf16_t* x, const bf16_t* w0, const bf16_t* w1,
                             const bf16_t* residual, bf16_t* y, int64_t m, int64_t k_in,
                             int64_t n_out, float* partial, hipStream_t st) {
    ProjParams p = {};
    p.hidden = x;
    p.row_idx = nullptr;
    p.w[0] = w0;
    p.w[1] = w1;
    p.out[0] = y;
    p.cs = nullptr;
    p.m = (int)m;
    p.hid = (int)k_in;
    const int nft = (int)(n_out / (mode == kProjGated ? T / 2 : T));
    p.tile_begin[0] = 0;
    p.tile_begin[1] = p.tile_begin[2] = p.tile_begin[3] = nft;
    p.partial = partial;
    p.n_ksplit = 1;
    p.residual = residual;
    p.n_out = (int)n_out;
    return mode == kProjGated ? launch_tiles<kProjGated>(p, st) : launch_tiles<kProjPlain>(p, st);
}

}  // namespace pkv
