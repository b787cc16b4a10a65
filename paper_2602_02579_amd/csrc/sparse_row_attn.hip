// Step 5: causal attention of the recomputed rows (selected context tokens
// and user-query tokens) over the whole updated cache.
// (Paper: Sec. 4.3 Stage II, complete recomputation but only for the
// selected tokens; Sec. 5.3, this attention dominates the cost; Eq. 1.)
//
//   out[i,h] = sum_{t <= row_pos[i]} softmax_t(q[i,h] . K[t,g(h)] * scale) V[t,g(h)]
#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <functional>
#include <mutex>
#include <queue>
#include <vector>

#include "attn_common.h"

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


// ---------------------------------------------------------------------------
// MFMA kernel: bf16 storage, head_dim 64 or 128, group size G <= 16.
//
// A workgroup (4 waves) owns a tile of BM = 256/G consecutive rows of one kv
// head g and the G query heads that read it: 256 "columns" (row, head), 64
// per wave.  It walks the keys 0 .. max position of the tile in steps of 64,
// staging K [64 keys x D] and V^T [D x 64 keys] tiles through double-buffered
// LDS.  Everything is computed transposed so that the softmax statistics of a
// column live in one lane (pair) and the probabilities feed the second MFMA
// straight from the accumulator registers:
//     S^T [keys x cols] = K  (A, from LDS)  x  Q^T (B, held in registers)
//     O^T [D    x cols] = V^T(A, from LDS)  x  P^T (B, the S^T accumulators)
// With v_mfma_f32_32x32x16_bf16 the accumulator of lane l holds column l%32
// and rows 8*(r/4) + 4*(l/32) + r%4, r = 0..15, while a B operand wants the 8
// contraction indices 8*(l/32) .. +7.  Reading K row swap_bits23(i) for A row
// i makes accumulator register r of lane half hh hold key 16*(r/8) + 8*hh +
// r%8 of the 32-key block, so registers 0..7 (8..15) are exactly the B operand
// of the first (second) 16 keys and V^T is read with plain contiguous keys.
// V^T comes from a transposed copy of the value cache made by a streaming
// pre-pass into the workspace.
//
// The same kernel with PV switched off and the key range split over
// blockIdx-encoded splits produces the per-column (max, sum) partials that
// the query-score call needs for its normalisers.  For head_dim 128 the
// attention proper runs in the software-pipelined kernel of
// sparse_row_attn_dma.hip; this one serves head_dim 64 and the partials.
// ---------------------------------------------------------------------------

template <int D>
struct AttnLds {
    static constexpr int kStride = D + 8;    // bf16 elements per K row
    static constexpr int vStride = kBN + 8;  // bf16 elements per V^T row
    static constexpr int kElems = kBN * kStride;
    static constexpr int vElems = D * vStride;
    static constexpr size_t bytes = 2 * (size_t)(kElems + vElems) * sizeof(bf16_t);
};

template <int D, bool kPV>
__global__ __launch_bounds__(kAttnThreads) void attn_mfma_kernel(AttnParams p) {
    typedef AttnLds<D> L;
    constexpr int KC = D / 16;               // contraction chunks of QK^T
    constexpr int DB = D / 32;               // 32-row blocks of O^T
    constexpr int CH = D * kBN / 8 / kAttnThreads;  // 16-byte chunks per thread per tile
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* k_lds = reinterpret_cast<bf16_t*>(smem_raw);            // [2][kElems]
    bf16_t* v_lds = k_lds + 2 * L::kElems;                          // [2][vElems]
    __shared__ int s_red[2][kAttnThreads / 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int hh = lane >> 5;
    const int l32 = lane & 31;

    // work item: kv head (fastest, so that a head stays on one XCD when
    // hkv == 8), key split, row tile (heaviest tiles first)
    // normally one work item per workgroup; the repair pass (p.flags set) is launched
    // with a small grid whose workgroups walk over all items and skip the unmarked ones;
    // the count of marked tiles sits behind the flags, and is zero almost always
    if (p.flags && p.flags[p.n_tiles * p.hkv] == 0) return;
    for (int wg0 = blockIdx.x; wg0 < p.n_tiles * p.n_splits * p.hkv; wg0 += gridDim.x) {
    int wg = wg0;
    const int g = wg % p.hkv;
    wg /= p.hkv;
    const int split = wg % p.n_splits;
    const int tile = p.n_tiles - 1 - wg / p.n_splits;
    // repair pass: only the tiles that the pipelined kernel marked
    if (p.flags && p.flags[tile * p.hkv + g] == 0) continue;

    // ---- my two columns ----------------------------------------------------
    int limit[2], row[2], head[2];
    bool valid[2];
    int lmax = -1, lmin = 0x7fffffff;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int col = wave * 64 + cb * 32 + l32;
        const int rl = col / p.group;
        row[cb] = tile * p.bm + rl;
        head[cb] = g * p.group + col % p.group;
        valid[cb] = rl < p.bm && row[cb] < p.m;
        limit[cb] = -1;
        if (valid[cb]) {
            limit[cb] = p.fixed_limit >= 0 ? p.fixed_limit : p.row_pos[row[cb]];
            lmax = max(lmax, limit[cb]);
            lmin = min(lmin, limit[cb]);
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        lmax = max(lmax, __shfl_xor(lmax, o, 64));
        lmin = min(lmin, __shfl_xor(lmin, o, 64));
    }
    if (lane == 0) s_red[0][wave] = lmax;
    __syncthreads();
    int tile_max = -1;
#pragma unroll
    for (int w = 0; w < kAttnThreads / 64; ++w) tile_max = max(tile_max, s_red[0][w]);
    const int wave_min = lmin;  // smallest limit among this wave's valid columns

    const int key_begin = split * p.split_len;
    const int key_end = min(min(tile_max + 1, p.n_keys), key_begin + p.split_len);

    // ---- Q as B operands, straight from global memory -------------------------
    bf16x8 qreg[2][KC];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const bf16_t* qp = p.q + ((int64_t)row[cb] * p.hq + head[cb]) * D + hh * 8;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            if (valid[cb]) {
                qreg[cb][kc] = *reinterpret_cast<const bf16x8*>(qp + kc * 16);
            } else {
                for (int j = 0; j < 8; ++j) qreg[cb][kc][j] = (bf16_t)0.0f;
            }
        }
    }

    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};
    // state at the context boundary (p.ctx_keys, a multiple of the key tile), for the
    // log-sum-exp over the context keys alone; NaN marks "boundary not reached"
    float m_ctx[2] = {0.f, 0.f}, l_ctx[2] = {-1.f, -1.f};
    f32x16 o_acc[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[db][cb][r] = 0.f;

    const int n_iter = key_end > key_begin ? (key_end - key_begin + kBN - 1) / kBN : 0;

    // ---- global -> register -> LDS staging --------------------------------------
    uint4 stage_k[CH], stage_v[CH];
    auto load_tile = [&](int t0) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = tid + kAttnThreads * i;
            const int key = c / (D / 8), dch = c % (D / 8);
            const int kk = min(t0 + key, p.n_keys - 1);
            stage_k[i] = *reinterpret_cast<const uint4*>(
                p.k + ((int64_t)kk * p.hkv + g) * D + dch * 8);
            if (kPV) {
                if (p.v) {
                    // no V^T copy was made (the pipelined kernel read the cache as it is):
                    // the same piece of the value row, transposed on its way into LDS.  Rows
                    // past the cache repeat its last row; their probabilities are zero.
                    stage_v[i] = *reinterpret_cast<const uint4*>(
                        p.v + ((int64_t)kk * p.hkv + g) * D + dch * 8);
                } else {
                    const int d = c / (kBN / 8), kch = c % (kBN / 8);
                    stage_v[i] = *reinterpret_cast<const uint4*>(
                        p.vt + ((int64_t)g * D + d) * p.n_pad + t0 + kch * 8);
                }
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = tid + kAttnThreads * i;
            const int key = c / (D / 8), dch = c % (D / 8);
            *reinterpret_cast<uint4*>(k_lds + buf * L::kElems + key * L::kStride + dch * 8) =
                stage_k[i];
            if (kPV) {
                if (p.v) {
                    const bf16x8 e = __builtin_bit_cast(bf16x8, stage_v[i]);
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        v_lds[buf * L::vElems + (dch * 8 + j) * L::vStride + key] = e[j];
                } else {
                    const int d = c / (kBN / 8), kch = c % (kBN / 8);
                    *reinterpret_cast<uint4*>(v_lds + buf * L::vElems + d * L::vStride + kch * 8) =
                        stage_v[i];
                }
            }
        }
    };

    // A-row i of a 32-key block reads key swap_bits23(i) of that block
    const int prow = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);

    if (n_iter > 0) {
        load_tile(key_begin);
        store_tile(0);
    }
    __syncthreads();

    for (int it = 0; it < n_iter; ++it) {
        const int t0 = key_begin + it * kBN;
        const int buf = it & 1;
        if (it + 1 < n_iter) load_tile(t0 + kBN);

        // ---- S^T = K Q^T ---------------------------------------------------------
        f32x16 s_acc[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s_acc[kb][cb][r] = 0.f;
        const bf16_t* kt = k_lds + buf * L::kElems + prow * L::kStride + hh * 8;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(kt + kc * 16);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(kt + 32 * L::kStride + kc * 16);
            s_acc[0][0] = mfma32(a0, qreg[0][kc], s_acc[0][0]);
            s_acc[0][1] = mfma32(a0, qreg[1][kc], s_acc[0][1]);
            s_acc[1][0] = mfma32(a1, qreg[0][kc], s_acc[1][0]);
            s_acc[1][1] = mfma32(a1, qreg[1][kc], s_acc[1][1]);
        }

        // ---- online softmax, one column per lane pair (l, l ^ 32) -----------------
        const bool need_mask = t0 + kBN - 1 > wave_min;
        bf16x8 pb[4][2];  // P^T as B operands: [16-key chunk][column block]
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            if (need_mask) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = t0 + 32 * kb + 16 * (r / 8) + 8 * hh + (r % 8);
                        if (key > limit[cb]) s_acc[kb][cb][r] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_acc[kb][cb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[cb], mx);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float corr = exp2f((m_run[cb] - m_safe) * p.scale_log2);
            const float msc = m_safe * p.scale_log2;
            float rs = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = exp2f(s_acc[kb][cb][r] * p.scale_log2 - msc);
                    rs += e;
                    s_acc[kb][cb][r] = e;
                }
            rs += __shfl_xor(rs, 32, 64);
            l_run[cb] = l_run[cb] * corr + rs;
            m_run[cb] = m_new;
            if (kPV) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[db][cb][r] *= corr;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int j2 = 0; j2 < 2; ++j2)
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            pb[2 * kb + j2][cb][e] = (bf16_t)s_acc[kb][cb][8 * j2 + e];
            }
        }

        // ---- O^T += V^T P^T ---------------------------------------------------------
        if (kPV) {
            const bf16_t* vtile = v_lds + buf * L::vElems + l32 * L::vStride + hh * 8;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(
                        vtile + db * 32 * L::vStride + kk * 16);
                    o_acc[db][0] = mfma32(a, pb[kk][0], o_acc[db][0]);
                    o_acc[db][1] = mfma32(a, pb[kk][1], o_acc[db][1]);
                }
        }

        if (p.lse_ctx && t0 + kBN == p.ctx_keys) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                m_ctx[cb] = m_run[cb];
                l_ctx[cb] = l_run[cb];
            }
        }
        if (it + 1 < n_iter) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue -----------------------------------------------------------------
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        if (!valid[cb]) continue;
        const int64_t colg = (int64_t)row[cb] * p.hq + head[cb];
        if (p.part_ml) {
            if (hh == 0) {
                float* dst = p.part_ml + ((int64_t)split * p.m * p.hq + colg) * 2;
                dst[0] = m_run[cb];
                dst[1] = l_run[cb];
            }
        } else {
            if (kPV) {
                const float inv = 1.f / l_run[cb];
                bf16_t* op = p.out + colg * D + 4 * hh;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        bf16x4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            v[e] = (bf16_t)(o_acc[db][cb][4 * r4 + e] * inv);
                        *reinterpret_cast<bf16x4*>(op + db * 32 + r4 * 8) = v;
                    }
            }
            if (p.lse && hh == 0)
                p.lse[colg] = m_run[cb] * p.scale + logf(l_run[cb]);
            if (p.lse_ctx && hh == 0)   // tiles that end below the boundary: all they saw
                p.lse_ctx[colg] = l_ctx[cb] < 0.f ? m_run[cb] * p.scale + logf(l_run[cb])
                                                  : m_ctx[cb] * p.scale + logf(l_ctx[cb]);
        }
    }
    __syncthreads();   // LDS and s_red are reused by the next work item
    }
}

// V [n_keys, hkv, D] -> V^T [hkv, D, n_pad], zero for keys >= n_keys.
// 64 x 64 tiles through LDS; reads and writes are both 16-byte, coalesced.
__device__ __forceinline__ void transpose_v_tile(const bf16_t* __restrict__ v,
                                                 bf16_t* __restrict__ vt, int n_keys, int n_pad,
                                                 int hkv, int d, int bx, int by,
                                                 bf16_t (*tile)[64 + 2]) {
    const int t0 = bx * 64;
    const int c0 = by * 64;  // column in the flattened [hkv * D] axis
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + 256 * i;      // 512 chunks of 8 elements
        const int t = c / 8, dch = c % 8;
        bf16x8 val;
        if (t0 + t < n_keys) {
            val = *reinterpret_cast<const bf16x8*>(
                v + (int64_t)(t0 + t) * hkv * d + c0 + dch * 8);
        } else {
            for (int j = 0; j < 8; ++j) val[j] = (bf16_t)0.0f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) tile[dch * 8 + j][t] = val[j];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + 256 * i;
        const int dd = c / 8, tch = c % 8;
        bf16x8 val;
#pragma unroll
        for (int j = 0; j < 8; ++j) val[j] = tile[dd][tch * 8 + j];
        // flattened column c0 + dd = g * D + d  ->  row of V^T
        *reinterpret_cast<bf16x8*>(vt + (int64_t)(c0 + dd) * n_pad + t0 + tch * 8) = val;
    }
}

__global__ __launch_bounds__(256) void transpose_v_kernel(
    const bf16_t* __restrict__ v, bf16_t* __restrict__ vt, int n_keys, int n_pad,
    int hkv, int d, int* zero, int n_zero) {
    __shared__ bf16_t tile[64][64 + 2];
    // this pre-pass also clears what the attention kernel expects at zero: the count of
    // tiles marked for the repair pass, the work-queue counters and, when the keys are
    // split, the marks themselves
    if (zero && blockIdx.x == 0 && blockIdx.y == 0)
        for (int i = threadIdx.x; i < n_zero; i += 256) zero[i] = 0;
    transpose_v_tile(v, vt, n_keys, n_pad, hkv, d, blockIdx.x, blockIdx.y, tile);
}

// What the pipelined kernel expects at zero when no V^T pre-pass runs before it.
__global__ __launch_bounds__(256) void attn_clear_kernel(int* zero, int n_zero) {
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n_zero; i += gridDim.x * 256) zero[i] = 0;
}

bool mfma_attn_supported(const pkv_layer_cfg& cfg) {
    const int group = cfg.n_q_heads / cfg.n_kv_heads;
    return cfg.dtype == PKV_BF16 && (cfg.head_dim == 64 || cfg.head_dim == 128) &&
           group <= 16;
}

int64_t pad64(int64_t n) { return (n + 63) & ~(int64_t)63; }

// workspace: V^T [hkv, D, n_pad] (rounded up to 256 bytes), then one int per
// (row tile, kv head) for the repair pass, the count of marked tiles, and one work-queue
// counter per kv head
size_t attn_vt_bytes(const pkv_layer_cfg& cfg, int64_t n_keys) {
    const size_t b = (size_t)cfg.n_kv_heads * cfg.head_dim * pad64(n_keys) * sizeof(bf16_t);
    return (b + 255) & ~(size_t)255;
}
size_t attn_flag_bytes(const pkv_layer_cfg& cfg, int64_t m) {
    const int bm = 256 / (cfg.n_q_heads / cfg.n_kv_heads);
    // + marked count + one work-queue counter per kv head
    const size_t b = ((size_t)ceil_div(m, bm) * cfg.n_kv_heads + 1 + cfg.n_kv_heads) * sizeof(int);
    return (b + 255) & ~(size_t)255;
}
// partial results that a small kernel merges.
constexpr int kMaxCtxRanges = 32;   // ranges per tile when a boundary is forced

// ctx_keys > 0: a range boundary must sit exactly at ctx_keys (a multiple of 64), because
// the log-sum-exp over the keys below it is read off the per-range partial results.  The
// context is cut into as many equal ranges as the time estimate wants, rounded down to a
// divisor of its length in 64-key units; the keys behind it take further ranges of that
// length.  Returns false when that would take more than kMaxCtxRanges ranges.
bool attn_plan_splits_at(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m, int64_t ctx_keys,
                         int* n_splits, int* split_len);

// Estimated time (us) of the pipelined launch when every row tile's keys are cut into `sp`
// ranges, for one layout of the row limits (the limits live on the device; the host weighs
// two layouts): `spread` = rows in position order with limits evenly over the keys, so tile i
// of T reaches (i + 1) / T of them; otherwise every tile reaches all keys.  The launch is one
// workgroup per CU claiming jobs heaviest first, which the longest-processing-time rule
// models; a job costs its 64-key steps plus a fixed set-up (pipeline fill, output; with ranges
// also the fp32 partial result), fitted to measured launches of 640 to 6681 rows.
double attn_launch_estimate(int64_t tiles, int hkv, int64_t steps_full, int sp, bool spread,
                            int n_cu) {
    const double us_per_step = 1.68, job_fixed = 4.0 + (sp > 1 ? 8.0 : 0.0);
    const int64_t range_steps = (steps_full + sp - 1) / sp;
    std::vector<double> jobs;
    jobs.reserve((size_t)(tiles * sp * hkv));
    for (int64_t i = 0; i < tiles; ++i) {
        const int64_t reach = spread ? std::max<int64_t>(1, (i + 1) * steps_full / tiles)
                                     : steps_full;
        for (int s = 0; s < sp; ++s) {
            const int64_t st = std::min<int64_t>(range_steps, reach - (int64_t)s * range_steps);
            if (st <= 0) break;
            for (int g = 0; g < hkv; ++g) jobs.push_back(st * us_per_step + job_fixed);
        }
    }
    std::sort(jobs.begin(), jobs.end(), std::greater<double>());
    std::priority_queue<double, std::vector<double>, std::greater<double>> cu;
    for (int c = 0; c < n_cu; ++c) cu.push(0.0);
    double end = 0.0;
    for (double j : jobs) {
        const double t = cu.top() + j;
        cu.pop();
        cu.push(t);
        end = std::max(end, t);
    }
    return end;
}

// Key ranges per row tile for the pipelined kernel.  With few (kv head, row tile) pairs per
// CU the launch ends when its longest job does - Stage I's 128 query rows make 16 jobs for
// 256 CUs, an 8k context with 1702 rows 216 jobs whose longest is twice the mean - so the
// keys of every tile are cut into up to 16 ranges (at least 2048 keys each, multiples of 64);
// the jobs write normalised partial results that a small kernel merges.  The count minimises
// the estimated launch time (the two layouts above, weighted by the row count) plus what the ranges cost: the
// jobs write and the merge kernel reads the partial results a row has (about 2 TB/s, measured, plus
// a launch).  Plans are remembered per problem size.
void attn_plan_splits(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m, int* n_splits,
                      int* split_len) {
    const int bm = 256 / (cfg.n_q_heads / cfg.n_kv_heads);
    const int64_t tiles = ceil_div(m, bm);
    const int64_t jobs = tiles * cfg.n_kv_heads;
    *n_splits = 1;
    *split_len = (int)pad64(n_keys);
    if (cfg.head_dim != 128 || jobs >= 1024 || jobs <= 0) return;
    const int64_t most = std::min<int64_t>(16, n_keys / 2048);   // ranges of 2048 keys or more
    if (most < 2) return;

    // PKV_ATTN_RANGES=n in the environment (read once) asks for n ranges whatever the estimate
    // says, within the bounds above: for measuring the estimate against the clock
    static const int forced = [] {
        const char* e = std::getenv("PKV_ATTN_RANGES");
        return e ? std::atoi(e) : 0;
    }();
    if (forced > 0) {
        const int64_t sp = std::min<int64_t>(forced, most);
        if (sp <= 1) return;
        const int64_t len = pad64(ceil_div(n_keys, sp));
        *split_len = (int)len;
        *n_splits = (int)ceil_div(n_keys, len);
        return;
    }
    struct Plan { int64_t n_keys, m; int hq, hkv, want; };
    static std::mutex mu;
    static std::vector<Plan> cache;
    int64_t want = 0;
    {
        std::lock_guard<std::mutex> lock(mu);
        for (const Plan& c : cache)
            if (c.n_keys == n_keys && c.m == m && c.hq == cfg.n_q_heads && c.hkv == cfg.n_kv_heads)
                want = c.want;
    }
    if (want == 0) {
        const int n_cu = 256;
        const int64_t steps_full = ceil_div(n_keys, 64);
        const double out_elems = (double)m * cfg.n_q_heads * cfg.head_dim;
        // a handful of rows are the user query, which sees the whole cache; thousands of rows
        // are selected context rows, whose positions cannot help being spread
        const double w_full = std::min(1.0, std::max(0.0, (768.0 - (double)m) / 640.0));
        double best = 1e30;
        for (int64_t sp = 1; sp <= most; ++sp) {
            const double run =
                (1.0 - w_full) * attn_launch_estimate(tiles, cfg.n_kv_heads, steps_full, (int)sp,
                                                      true, n_cu) +
                w_full * attn_launch_estimate(tiles, cfg.n_kv_heads, steps_full, (int)sp, false,
                                              n_cu);
            // partial results: a row has (sp + 1) / 2 (spread) or sp (full) of them, fp32, written
            // by the jobs and read back by the merge, which also writes the output.  Measured
            // against unsplit launches (6681 rows in 2 ranges, 3404 in 4, 1702 in 2) the whole
            // detour moves at about 2 TB/s.
            const double ranges = w_full * sp + (1.0 - w_full) * 0.5 * (sp + 1);
            const double merge = sp == 1 ? 0.0
                : 5.0 + (out_elems * 4.0 * ranges * 2.0 + out_elems * 2.0) / 2.0e6;
            if (run + merge < best - 1e-9) {
                best = run + merge;
                want = sp;
            }
        }
        std::lock_guard<std::mutex> lock(mu);
        if (cache.size() >= 64) cache.erase(cache.begin());
        cache.push_back(Plan{n_keys, m, cfg.n_q_heads, cfg.n_kv_heads, (int)want});
    }
    if (want <= 1) return;
    const int64_t len = pad64(ceil_div(n_keys, want));
    *split_len = (int)len;
    *n_splits = (int)ceil_div(n_keys, len);
}
bool attn_plan_splits_at(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m, int64_t ctx_keys,
                         int* n_splits, int* split_len) {
    int want = 1, len = 0;
    attn_plan_splits(cfg, n_keys, m, &want, &len);
    const int64_t units = ctx_keys / 64;
    for (int64_t s = std::min<int64_t>(std::max(want, 1), units); s >= 1; --s) {
        if (units % s) continue;
        const int64_t l = ctx_keys / s;
        const int64_t total = ceil_div(n_keys, l);
        if (total > kMaxCtxRanges) continue;
        *split_len = (int)l;
        *n_splits = (int)total;
        return true;
    }
    return false;
}

size_t attn_partial_bytes(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m,
                          int64_t ctx_keys = 0) {
    int n_splits, split_len;
    if (ctx_keys > 0) {
        if (!attn_plan_splits_at(cfg, n_keys, m, ctx_keys, &n_splits, &split_len)) return 0;
    } else {
        attn_plan_splits(cfg, n_keys, m, &n_splits, &split_len);
    }
    if (n_splits <= 1) return 0;
    const size_t cols = (size_t)m * cfg.n_q_heads;
    return (size_t)n_splits * cols * (cfg.head_dim + 1) * sizeof(float);
}

template <int D, bool kPV>
pkv_status launch_attn_mfma(const AttnParams& p, hipStream_t st) {
    static std::atomic<bool> configured{false};   // set twice at worst: the calls are idempotent  // per process; the attribute is per function
    auto kern = attn_mfma_kernel<D, kPV>;
    if (!configured.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)AttnLds<D>::bytes) != hipSuccess)
            return PKV_ERR_LAUNCH;
        configured.store(true, std::memory_order_release);
    }
    int64_t grid = (int64_t)p.n_tiles * p.n_splits * p.hkv;
    if (p.flags && grid > 256) grid = 256;   // repair pass: one resident workgroup per CU
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kAttnThreads), AttnLds<D>::bytes,
                       st, p);
    return launch_status();
}

}  // namespace

size_t sparse_row_attn_ws_bytes(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m,
                                int64_t ctx_keys) {
    if (!mfma_attn_supported(cfg)) return 0;
    return attn_vt_bytes(cfg, n_keys) + attn_flag_bytes(cfg, m) +
           attn_partial_bytes(cfg, n_keys, m, ctx_keys);
}

bool sparse_row_attn_ctx_lse_supported(const pkv_layer_cfg& cfg, int64_t n_keys, int64_t m,
                                       int64_t ctx_keys) {
    int a, b;
    return mfma_attn_supported(cfg) && cfg.head_dim == 128 && ctx_keys > 0 &&
           ctx_keys % 64 == 0 && ctx_keys <= n_keys &&
           attn_plan_splits_at(cfg, n_keys, m, ctx_keys, &a, &b);
}

// Per-column (max, sum) partials of softmax(q k^T * scale) over keys
// 0 .. n_ctx-1, split over the keys; used by the query-score call.
// part_ml: [n_splits, nq*hq, 2].
pkv_status launch_attn_lse_partials(const pkv_layer_cfg& cfg, const void* q,
                                    const void* k, int64_t nq, int64_t n_ctx,
                                    float scale, int n_splits, int split_len,
                                    float* part_ml, hipStream_t st) {
    AttnParams p = {};
    p.q = (const bf16_t*)q;
    p.k = (const bf16_t*)k;
    p.part_ml = part_ml;
    p.m = (int)nq;
    p.n_keys = (int)n_ctx;
    p.n_pad = (int)pad64(n_ctx);
    p.hq = cfg.n_q_heads;
    p.hkv = cfg.n_kv_heads;
    p.group = cfg.n_q_heads / cfg.n_kv_heads;
    p.bm = 256 / p.group;
    p.n_tiles = (int)ceil_div(nq, p.bm);
    p.n_splits = n_splits;
    p.split_len = split_len;
    p.fixed_limit = (int)n_ctx - 1;
    p.scale = scale;
    p.scale_log2 = scale * 1.4426950408889634f;
    return cfg.head_dim == 128 ? launch_attn_mfma<128, false>(p, st)
                               : launch_attn_mfma<64, false>(p, st);
}

pkv_status launch_sparse_row_attn(const pkv_layer_cfg& cfg, const void* q,
                                  const void* k_cache, const void* v_cache,
                                  const int32_t* row_pos, void* out,
                                  float* lse_out, int64_t m, int64_t n_keys,
                                  float scale, void* ws, hipStream_t st,
                                  int64_t ctx_keys, float* lse_ctx_out) {
    if (m == 0) return PKV_OK;
    const int d = cfg.head_dim;
    if (lse_ctx_out && !sparse_row_attn_ctx_lse_supported(cfg, n_keys, m, ctx_keys))
        return PKV_ERR_UNSUPPORTED;
    if (mfma_attn_supported(cfg)) {
        const int n_pad = (int)pad64(n_keys);
        bf16_t* vt = (bf16_t*)ws;
        int* const ints = reinterpret_cast<int*>((unsigned char*)ws + attn_vt_bytes(cfg, n_keys));
        const int n_flags =
            (int)ceil_div(m, 256 / (cfg.n_q_heads / cfg.n_kv_heads)) * cfg.n_kv_heads;
        int n_splits = 1, split_len = n_pad;
        if (lse_ctx_out)
            attn_plan_splits_at(cfg, n_keys, m, ctx_keys, &n_splits, &split_len);
        else
            attn_plan_splits(cfg, n_keys, m, &n_splits, &split_len);
        // cleared by the pre-pass: marked count + queue counters, and the marks when split
        int* zero = d == 128 ? (n_splits > 1 ? ints : ints + n_flags) : nullptr;
        const int n_zero = (n_splits > 1 ? n_flags : 0) + 1 + cfg.n_kv_heads;
        // The eight-wave pipelined kernel can transpose the values on their way out of LDS
        // instead of reading a V^T copy made here.  Its loop then issues half as many bytes per
        // LDS instruction and needs ~2 % more clocks (about 1 % more time at the clock the part
        // grants: 131k keys x 26470 rows 21.6 -> 21.8 ms); the copy costs its bytes at ~5.5 TB/s
        // plus a launch, and doing without it costs one small launch (a fill kernel for the
        // counters that the pre-pass otherwise clears).  The copy is skipped when that is the
        // cheaper side, which it is for everything but the largest launches (measured, copy ->
        // no copy: 128 rows over 32k keys 106 -> 85 us, 1766 rows 487 -> 470 us, 6681 rows
        // 1496 -> 1486 us, 13235 rows 2785 -> 2784 us).
        bool nat_v = false;
        if (d == 128) {
            const int src = attn_dma128_v_source();
            if (src < 0) {
                const int bm = 256 / (cfg.n_q_heads / cfg.n_kv_heads);
                const double copy_us = 3.0 + (double)n_pad * cfg.n_kv_heads * d * 4.0 / 5.5e6;
                const double main_us = 1.68 * (double)ceil_div(m, bm) * cfg.n_kv_heads *
                                       (double)(n_pad / 64) * (m > 768 ? 0.5 : 1.0) / 256.0;
                nat_v = copy_us - 4.0 > 0.012 * main_us;
            } else {
                nat_v = src == 0;
            }
        }
        if (nat_v)
            hipLaunchKernelGGL(attn_clear_kernel, dim3((unsigned)std::min(64, (n_zero + 255) / 256)),
                               dim3(256), 0, st, zero, n_zero);
        else
            hipLaunchKernelGGL(transpose_v_kernel,
                               dim3((unsigned)(n_pad / 64), (unsigned)(cfg.n_kv_heads * d / 64)),
                               dim3(256), 0, st, (const bf16_t*)v_cache, vt, (int)n_keys, n_pad,
                               cfg.n_kv_heads, d, zero, n_zero);
        if (launch_status() != PKV_OK) return PKV_ERR_LAUNCH;
        AttnParams p = {};
        p.q = (const bf16_t*)q;
        p.k = (const bf16_t*)k_cache;
        p.vt = vt;
        p.v = nat_v ? (const bf16_t*)v_cache : nullptr;
        p.row_pos = row_pos;
        p.out = (bf16_t*)out;
        p.lse = lse_out;
        p.m = (int)m;
        p.n_keys = (int)n_keys;
        p.n_pad = n_pad;
        p.hq = cfg.n_q_heads;
        p.hkv = cfg.n_kv_heads;
        p.group = cfg.n_q_heads / cfg.n_kv_heads;
        p.bm = 256 / p.group;
        p.n_tiles = (int)ceil_div(m, p.bm);
        p.n_splits = 1;
        p.split_len = n_pad;
        p.fixed_limit = -1;
        p.scale = scale;
        p.scale_log2 = scale * 1.4426950408889634f;
        if (d != 128) return launch_attn_mfma<64, true>(p, st);
        // pipelined kernel with a fixed softmax reference per column, then the exact
        // kernel on the tiles it marked (normally none: those workgroups exit at once)
        p.flags = ints;
        p.queue = p.flags + p.n_tiles * p.hkv + 1;
        p.dma_splits = n_splits;
        p.dma_split_len = split_len;
        p.lse_ctx = lse_ctx_out;
        p.ctx_keys = (int)ctx_keys;
        if (n_splits > 1) {
            p.part_o = reinterpret_cast<float*>((unsigned char*)ws + attn_vt_bytes(cfg, n_keys) +
                                                attn_flag_bytes(cfg, m));
            p.part_lse = p.part_o + (size_t)n_splits * m * cfg.n_q_heads * d;
        }
        const pkv_status rc = launch_attn_dma128(p, st);
        if (rc != PKV_OK) return rc;
        // (p.v set: the exact kernel, too, reads the cache as it is for the tiles it redoes)
        return launch_attn_mfma<128, true>(p, st);
    }
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
