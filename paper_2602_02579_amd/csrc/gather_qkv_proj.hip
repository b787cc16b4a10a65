// Step 4a: gather the hidden rows of the selected and the query tokens,
// project them to Q/K/V and rotate Q and K to each row's own position.
// (Paper: Algorithm 1, "Recompute KV cache at layer l" and "Calculate user
// query KV cache"; Appendix E: hidden states and positions are pruned to the
// selected tokens before the forward pass.)
//
// out[i, head, :] = R(row_pos[i]) (W_head x_i),  x_i = hidden[row_idx[i]]
// for the Hq query heads, the Hkv key heads, and (without R) the Hkv value
// heads; fp32 accumulation; one rounding after the rotation.
#include "proj_common.h"

namespace pkv {

namespace {

// ---------------------------------------------------------------------------
// Generic kernel: any head_dim (multiple of 16), fp32 or bf16 storage, plain
// fp32 FMAs.  A block owns 16 gathered rows of one output head; a work item
// is one (row, pair index i) and produces output elements i and i + D/2, so
// the rotation is local to the thread.
// ---------------------------------------------------------------------------
// Block variants: bias[3] are additive biases of the three projections, gain[2] the
// gains of an RMS norm over head_dim applied to every head of Q and K before the
// rotation (null = absent).  The norm needs the whole head of a row: the squares go
// through LDS and every work item adds up its row's D/2 partial sums in a fixed order.
struct ProjExtra {
    const void* bias[3];
    const void* gain[2];
    float eps;
    const int32_t* dst_row;   // fused cache update of K and V (null = plain outputs)
};

template <typename T>
__global__ __launch_bounds__(256) void qkv_proj_generic(
    const T* __restrict__ hidden, const int32_t* __restrict__ row_idx,
    const int32_t* __restrict__ row_pos, const T* __restrict__ wq,
    const T* __restrict__ wk, const T* __restrict__ wv, T* __restrict__ q_out,
    T* __restrict__ k_out, T* __restrict__ v_out, int m, int hq, int hkv, int d,
    int hid, RopeTable tab, ProjExtra ex) {
    constexpr int V = Vec16<T>::N;
    constexpr int kMaxItems = 16 * kMaxHalfDim / 256;   // work items per thread
    typedef typename Vec16<T>::type vec_t;
    __shared__ float s_sq[16 * kMaxHalfDim];
    const int head = blockIdx.y;  // [0,hq) Q, [hq,hq+hkv) K, [hq+hkv,hq+2hkv) V
    const T* w;
    T* out;
    int heads_out, head_local, mat;
    if (head < hq) {
        w = wq; out = q_out; heads_out = hq; head_local = head; mat = 0;
    } else if (head < hq + hkv) {
        w = wk; out = k_out; heads_out = hkv; head_local = head - hq; mat = 1;
    } else {
        w = wv; out = v_out; heads_out = hkv; head_local = head - hq - hkv; mat = 2;
    }
    if (out == nullptr) return;   // uniform over the block
    const bool rotate = mat != 2;
    const T* bias = static_cast<const T*>(ex.bias[mat]);
    const T* gain = mat != 2 ? static_cast<const T*>(ex.gain[mat]) : nullptr;
    const int half = d / 2;
    const int row0 = blockIdx.x * 16;
    float va[kMaxItems], vb[kMaxItems];
#pragma unroll
    for (int it = 0; it < kMaxItems; ++it) {
        const int item = threadIdx.x + it * 256;
        va[it] = vb[it] = 0.f;
        if (item >= 16 * half) continue;
        const int r = row0 + item / half;
        const int i = item % half;
        if (r < m) {
            const int64_t src_row = row_idx ? row_idx[r] : r;
            const T* x = hidden + src_row * hid;
            const T* wa = w + ((int64_t)head_local * d + i) * hid;
            const T* wb = wa + (int64_t)half * hid;
            float a = 0.f, b = 0.f;
            for (int c = 0; c < hid; c += V) {
                const vec_t xv = *reinterpret_cast<const vec_t*>(x + c);
                const vec_t av = *reinterpret_cast<const vec_t*>(wa + c);
                const vec_t bv = *reinterpret_cast<const vec_t*>(wb + c);
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    const float xf = Elem<T>::to_f32(xv[j]);
                    a += xf * Elem<T>::to_f32(av[j]);
                    b += xf * Elem<T>::to_f32(bv[j]);
                }
            }
            if (bias) {
                a += Elem<T>::load(bias + head_local * d + i);
                b += Elem<T>::load(bias + head_local * d + i + half);
            }
            va[it] = a;
            vb[it] = b;
        }
        if (gain) s_sq[item] = va[it] * va[it] + vb[it] * vb[it];
    }
    if (gain) __syncthreads();    // uniform: gain depends on the block's head only
#pragma unroll
    for (int it = 0; it < kMaxItems; ++it) {
        const int item = threadIdx.x + it * 256;
        if (item >= 16 * half) continue;
        const int r = row0 + item / half;
        const int i = item % half;
        if (r >= m) continue;
        float a = va[it], b = vb[it];
        if (gain) {
            float ss = 0.f;
            const float* sq = s_sq + (item / half) * half;
            for (int t = 0; t < half; ++t) ss += sq[t];
            const float rn = 1.0f / sqrtf(ss / (float)d + ex.eps);
            a = a * rn * Elem<T>::load(gain + i);
            b = b * rn * Elem<T>::load(gain + i + half);
        }
        float ra = a, rb = b;
        if (rotate) {
            float sn, cs;
            rope_sincos((double)row_pos[r], tab.inv_freq[i], &sn, &cs);
            ra = a * cs - b * sn;
            rb = b * cs + a * sn;
        }
        const int64_t orow = (mat != 0 && ex.dst_row) ? ex.dst_row[r] : r;
        T* o = out + (orow * heads_out + head_local) * d;
        o[i] = Elem<T>::from_f32(ra);
        o[i + half] = Elem<T>::from_f32(rb);
    }
}


// ---------------------------------------------------------------------------
// MFMA kernel: bf16 storage, head_dim 64 or 128, hidden a multiple of 32.
//
// C[256 rows x 128 cols] per workgroup, contraction in steps of 32 through
// double-buffered LDS, v_mfma_f32_32x32x16_bf16.  Both operands have the
// contraction dimension contiguous in memory (x rows and weight rows), which
// is exactly what the A and B operands want (8 consecutive k per lane).
// The gather costs nothing extra: the A-tile loader reads row row_idx[i].
//
// The 4 waves sit 2 x 2 over the tile; a wave owns 128 rows and two 32-column
// blocks chosen so that block 1 is the rotary partner (i + D/2) of block 0.
// The accumulator of a lane then holds both elements of every rotary pair and
// the rotation happens in registers, with cos/sin read from a small table
// [m, D/2] that a pre-pass fills (one sincos per (row, i) for all heads).
// ---------------------------------------------------------------------------

constexpr int kGM = 256, kGN = 128, kGK = 32;
constexpr int kAStride = kGK + 8;  // bf16 elements per LDS row (80 bytes)

__global__ void rope_table_kernel(const int32_t* __restrict__ row_pos, int m, int half,
                                  RopeTable tab, float2* __restrict__ cs) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)m * half) return;
    const int r = (int)(idx / half), i = (int)(idx % half);
    float sn, c;
    rope_sincos((double)row_pos[r], tab.inv_freq[i], &sn, &c);
    cs[idx] = make_float2(c, sn);
}

template <int D>
__global__ __launch_bounds__(256, 2) void qkv_proj_mfma(ProjParams p) {
    __shared__ __align__(16) bf16_t a_lds[2][kGM * kAStride];
    __shared__ __align__(16) bf16_t b_lds[2][kGN * kAStride];
    constexpr int HALF = D / 2;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int hh = lane >> 5, l32 = lane & 31;
    const int wm = wave >> 1, wn = wave & 1;

    // which matrix and which 128 output columns
    const int ct = blockIdx.x;
    int mat = 0;
    if (ct >= p.tile_begin[1]) mat = 1;
    if (ct >= p.tile_begin[2]) mat = 2;
    const int col0 = (ct - p.tile_begin[mat]) * kGN;   // first output feature of the tile
    const bf16_t* w = p.w[mat];
    bf16_t* out = p.out[mat];
    const int heads_out = mat == 0 ? p.hq : p.hkv;
    const int row0 = blockIdx.y * kGM;

    // ---- loaders: A 256 x 32 (4 chunks / thread), B 128 x 32 (2 chunks / thread)
    const bf16_t* a_src[4];
    int a_dst[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i;
        const int r = c >> 2, kch = c & 3;
        int gr = row0 + r;
        if (gr >= p.m) gr = p.m - 1;
        const int64_t src_row = p.row_idx ? p.row_idx[gr] : gr;
        a_src[i] = p.hidden + src_row * p.hid + kch * 8;
        a_dst[i] = r * kAStride + kch * 8;
    }
    const bf16_t* b_src[2];
    int b_dst[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + 256 * i;
        const int r = c >> 2, kch = c & 3;
        b_src[i] = w + (int64_t)(col0 + r) * p.hid + kch * 8;
        b_dst[i] = r * kAStride + kch * 8;
    }
    uint4 sa[4], sb[2];
    auto load_stage = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) sa[i] = *reinterpret_cast<const uint4*>(a_src[i] + k0);
#pragma unroll
        for (int i = 0; i < 2; ++i) sb[i] = *reinterpret_cast<const uint4*>(b_src[i] + k0);
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(&a_lds[buf][a_dst[i]]) = sa[i];
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<uint4*>(&b_lds[buf][b_dst[i]]) = sb[i];
    };

    // wave's column blocks: block 1 is the rotary partner of block 0
    // D = 128: the tile is one head; wave wn owns i in [32 wn, 32 wn + 32) and i + 64
    // D = 64 : the tile is two heads; wave wn owns head wn, i in [0, 32) and i + 32
    const int cb0 = D == 128 ? wn * 32 : wn * 64;
    const int cb1 = cb0 + HALF;

    f32x16 acc[4][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    const int n_k = p.hid / kGK;
    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int kt = 0; kt < n_k; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < n_k) load_stage((kt + 1) * kGK);
        const bf16_t* ap = &a_lds[buf][(wm * 128 + l32) * kAStride + hh * 8];
        const bf16_t* bp = &b_lds[buf][l32 * kAStride + hh * 8];
#pragma unroll
        for (int ks = 0; ks < kGK / 16; ++ks) {
            bf16x8 a[4], b[2];
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
                a[mb] = *reinterpret_cast<const bf16x8*>(ap + mb * 32 * kAStride + ks * 16);
            b[0] = *reinterpret_cast<const bf16x8*>(bp + cb0 * kAStride + ks * 16);
            b[1] = *reinterpret_cast<const bf16x8*>(bp + cb1 * kAStride + ks * 16);
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                acc[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb], b[0], acc[mb][0], 0, 0, 0);
                acc[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb], b[1], acc[mb][1], 0, 0, 0);
            }
        }
        if (kt + 1 < n_k) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: rotate pairs in registers, round once, store -----------------
    if (out == nullptr) return;
    const int head = (col0 + cb0) / D;            // output head of this wave's columns
    const int i = (col0 + cb0) % D + l32;         // pair index in [0, D/2)
    const bool rotate = mat != 2;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + wm * 128 + mb * 32 + 8 * (r / 4) + 4 * hh + (r % 4);
            if (row >= p.m) continue;
            float a = acc[mb][0][r], b = acc[mb][1][r];
            if (rotate) {
                const float2 t = p.cs[(int64_t)row * HALF + i];
                const float ra = a * t.x - b * t.y;
                const float rb = b * t.x + a * t.y;
                a = ra;
                b = rb;
            }
            const int64_t orow = (mat != 0 && p.dst_row) ? p.dst_row[row] : row;
            bf16_t* o = out + (orow * heads_out + head) * D + i;
            o[0] = (bf16_t)a;
            o[HALF] = (bf16_t)b;
        }
}

bool mfma_proj_supported(const pkv_layer_cfg& cfg) {
    if (cfg.dtype != PKV_BF16 || cfg.hidden % kGK) return false;
    if (cfg.head_dim == 128) return true;
    return cfg.head_dim == 64 && cfg.n_q_heads % 2 == 0 && cfg.n_kv_heads % 2 == 0;
}

}  // namespace

size_t gather_qkv_proj_ws_bytes(const pkv_layer_cfg& cfg, int64_t m) {
    if (!mfma_proj_supported(cfg)) return 0;
    size_t b = (size_t)m * (cfg.head_dim / 2) * sizeof(float2);
    b = (b + 255) & ~(size_t)255;
    if (proj_dma128_supported(cfg, m)) b += proj_dma128_partial_bytes(cfg, m);
    return b;
}

pkv_status launch_gather_qkv_proj(const pkv_layer_cfg& cfg, const void* hidden,
                                  const int32_t* row_idx, const int32_t* row_pos,
                                  const void* wq, const void* wk, const void* wv,
                                  const pkv_proj_variant* var, const int32_t* dst_row,
                                  void* q_out, void* k_out, void* v_out, int64_t m, void* ws,
                                  hipStream_t st) {
    if (m == 0) return PKV_OK;
    ProjExtra ex = {};
    ex.dst_row = dst_row;
    if (var) {
        ex.bias[0] = var->bq; ex.bias[1] = var->bk; ex.bias[2] = var->bv;
        ex.gain[0] = var->q_norm; ex.gain[1] = var->k_norm;
        ex.eps = var->norm_eps;
    }
    const bool extra = ex.bias[0] || ex.bias[1] || ex.bias[2] || ex.gain[0] || ex.gain[1];
    RopeTable tab;
    fill_rope_table(&tab, cfg.head_dim, (double)cfg.rope_theta);
    const int hq = cfg.n_q_heads, hkv = cfg.n_kv_heads;
    // the variants are built into the 256 x 256 tile kernel and the plain kernel; the older
    // 256 x 128 MFMA kernel (head_dim 64, odd head counts) does not have them
    if (mfma_proj_supported(cfg) && (!extra || proj_dma128_supported(cfg, m))) {
        const int d = cfg.head_dim, half = d / 2;
        float2* cs = (float2*)ws;
        const int64_t n_tab = m * half;
        hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)ceil_div(n_tab, 256)), dim3(256),
                           0, st, row_pos, (int)m, half, tab, cs);
        ProjParams p = {};
        p.hidden = (const bf16_t*)hidden;
        p.row_idx = row_idx;
        p.w[0] = (const bf16_t*)wq; p.w[1] = (const bf16_t*)wk; p.w[2] = (const bf16_t*)wv;
        p.out[0] = (bf16_t*)q_out; p.out[1] = (bf16_t*)k_out; p.out[2] = (bf16_t*)v_out;
        p.cs = cs;
        p.m = (int)m; p.hid = cfg.hidden; p.hq = hq; p.hkv = hkv;
        for (int i = 0; i < 3; ++i) p.bias[i] = (const bf16_t*)ex.bias[i];
        for (int i = 0; i < 2; ++i) p.norm_w[i] = (const bf16_t*)ex.gain[i];
        p.norm_eps = ex.eps;
        p.dst_row = dst_row;
        if (proj_dma128_supported(cfg, m)) {
            const int tq = q_out ? hq * d / kProjDmaTile : 0;
            const int tkv = k_out ? hkv * d / kProjDmaTile : 0;
            p.tile_begin[0] = 0;
            p.tile_begin[1] = tq;
            p.tile_begin[2] = tq + tkv;
            p.tile_begin[3] = tq + 2 * tkv;
            const size_t cs_bytes = ((size_t)m * half * sizeof(float2) + 255) & ~(size_t)255;
            p.partial = reinterpret_cast<float*>((unsigned char*)ws + cs_bytes);
            return launch_proj_dma128(p, st);
        }
        // column tiles: only the matrices whose outputs were asked for
        const int tq = q_out ? hq * d / kGN : 0;
        const int tkv = k_out ? hkv * d / kGN : 0;
        p.tile_begin[0] = 0;
        p.tile_begin[1] = tq;
        p.tile_begin[2] = tq + tkv;
        p.tile_begin[3] = tq + 2 * tkv;
        const dim3 grid((unsigned)p.tile_begin[3], (unsigned)ceil_div(m, kGM));
        if (d == 128) hipLaunchKernelGGL(qkv_proj_mfma<128>, grid, dim3(256), 0, st, p);
        else hipLaunchKernelGGL(qkv_proj_mfma<64>, grid, dim3(256), 0, st, p);
        return launch_status();
    }
    const dim3 grid((unsigned)ceil_div(m, 16), (unsigned)(hq + 2 * hkv));
    if (cfg.dtype == PKV_BF16) {
        hipLaunchKernelGGL(qkv_proj_generic<bf16_t>, grid, dim3(256), 0, st,
                           (const bf16_t*)hidden, row_idx, row_pos,
                           (const bf16_t*)wq, (const bf16_t*)wk, (const bf16_t*)wv,
                           (bf16_t*)q_out, (bf16_t*)k_out, (bf16_t*)v_out, (int)m,
                           hq, hkv, cfg.head_dim, cfg.hidden, tab, ex);
    } else {
        hipLaunchKernelGGL(qkv_proj_generic<float>, grid, dim3(256), 0, st,
                           (const float*)hidden, row_idx, row_pos,
                           (const float*)wq, (const float*)wk, (const float*)wv,
                           (float*)q_out, (float*)k_out, (float*)v_out, (int)m, hq,
                           hkv, cfg.head_dim, cfg.hidden, tab, ex);
    }
    return launch_status();
}

}  // namespace pkv
