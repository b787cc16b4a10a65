// Step 4a: gather the hidden rows of the selected and the query tokens,
// project them to Q/K/V and rotate Q and K to each row's own position.
// (Paper: Algorithm 1, "Recompute KV cache at layer l" and "Calculate user
// query KV cache"; Appendix E: hidden states and positions are pruned to the
// selected tokens before the forward pass.)
//
// out[i, head, :] = R(row_pos[i]) (W_head x_i),  x_i = hidden[row_idx[i]]
// for the Hq query heads, the Hkv key heads, and (without R) the Hkv value
// heads; fp32 accumulation; one rounding after the rotation.
#include "pkv_common.h"

namespace pkv {

namespace {

// ---------------------------------------------------------------------------
// Generic kernel: any head_dim (multiple of 16), fp32 or bf16 storage, plain
// fp32 FMAs.  A block owns 16 gathered rows of one output head; a work item
// is one (row, pair index i) and produces output elements i and i + D/2, so
// the rotation is local to the thread.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void qkv_proj_generic(
    const T* __restrict__ hidden, const int32_t* __restrict__ row_idx,
    const int32_t* __restrict__ row_pos, const T* __restrict__ wq,
    const T* __restrict__ wk, const T* __restrict__ wv, T* __restrict__ q_out,
    T* __restrict__ k_out, T* __restrict__ v_out, int m, int hq, int hkv, int d,
    int hid, RopeTable tab) {
    constexpr int V = Vec16<T>::N;
    typedef typename Vec16<T>::type vec_t;
    const int head = blockIdx.y;  // [0,hq) Q, [hq,hq+hkv) K, [hq+hkv,hq+2hkv) V
    const T* w;
    T* out;
    int heads_out, head_local;
    bool rotate;
    if (head < hq) {
        w = wq; out = q_out; heads_out = hq; head_local = head; rotate = true;
    } else if (head < hq + hkv) {
        w = wk; out = k_out; heads_out = hkv; head_local = head - hq; rotate = true;
    } else {
        w = wv; out = v_out; heads_out = hkv; head_local = head - hq - hkv; rotate = false;
    }
    if (out == nullptr) return;
    const int half = d / 2;
    const int row0 = blockIdx.x * 16;
    for (int item = threadIdx.x; item < 16 * half; item += 256) {
        const int r = row0 + item / half;
        const int i = item % half;
        if (r >= m) continue;
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
        float ra = a, rb = b;
        if (rotate) {
            float sn, cs;
            rope_sincos((double)row_pos[r], tab.inv_freq[i], &sn, &cs);
            ra = a * cs - b * sn;
            rb = b * cs + a * sn;
        }
        T* o = out + ((int64_t)r * heads_out + head_local) * d;
        o[i] = Elem<T>::from_f32(ra);
        o[i + half] = Elem<T>::from_f32(rb);
    }
}

}  // namespace

pkv_status launch_gather_qkv_proj(const pkv_layer_cfg& cfg, const void* hidden,
                                  const int32_t* row_idx, const int32_t* row_pos,
                                  const void* wq, const void* wk, const void* wv,
                                  void* q_out, void* k_out, void* v_out,
                                  int64_t m, hipStream_t st) {
    if (m == 0) return PKV_OK;
    RopeTable tab;
    fill_rope_table(&tab, cfg.head_dim, (double)cfg.rope_theta);
    const int hq = cfg.n_q_heads, hkv = cfg.n_kv_heads;
    const dim3 grid((unsigned)ceil_div(m, 16), (unsigned)(hq + 2 * hkv));
    if (cfg.dtype == PKV_BF16) {
        hipLaunchKernelGGL(qkv_proj_generic<bf16_t>, grid, dim3(256), 0, st,
                           (const bf16_t*)hidden, row_idx, row_pos,
                           (const bf16_t*)wq, (const bf16_t*)wk, (const bf16_t*)wv,
                           (bf16_t*)q_out, (bf16_t*)k_out, (bf16_t*)v_out, (int)m,
                           hq, hkv, cfg.head_dim, cfg.hidden, tab);
    } else {
        hipLaunchKernelGGL(qkv_proj_generic<float>, grid, dim3(256), 0, st,
                           (const float*)hidden, row_idx, row_pos,
                           (const float*)wq, (const float*)wk, (const float*)wv,
                           (float*)q_out, (float*)k_out, (float*)v_out, (int)m, hq,
                           hkv, cfg.head_dim, cfg.hidden, tab);
    }
    return launch_status();
}

}  // namespace pkv
