// Decode step of one CQIL group for a single new token (B*T == 1): five bandwidth-bound kernels and a merge.
//
//   1 qkv_rope   shared-input projection of all P layers (Eq.2's xW^Q, xW^K, xW^V applied to the one x_G of
//                Eq.3), fused with the attention RMSNorm (one statistic for the whole group, P gains), the
//                rotary embedding and the KV-cache append
//   2 attn       softmax(QK^T/sqrt(d_k))V over the P independent caches (cqil_attn.h)
//   3 oproj      per-layer Concat(heads)W^O
//   4 gateup     forms the P feed-forward inputs h_i = x + a_i + bypass window (Eq.4), their RMSNorm, the
//                gate/up projections and SwiGLU
//   5 down       one contraction over the K-concatenated Wdown: sum_i FFN_i, split along K
//   6 merge      x_out = x + sum_i a_i + sum of the K slices (Eq.3 / Eq.4)
//
// Every projection is a matrix-vector product streamed once from HBM in the tiled layout: a wave owns 16-row
// strips, each of its loads reads one contiguous 1 KiB tile, the input vector sits in LDS as fp32.  A unit of
// work is one strip (O, down) or the two strips that meet in an epilogue (the two halves of 16 rotary pairs; 16
// gate rows and their 16 up rows).  A workgroup of 8 waves takes 8 / ksplit units; with ksplit > 1 the waves of
// a unit split the k range and add their parts through LDS in a fixed order.
#include "cqil_attn.h"
#include "cqil_dev.h"
#include "cqil_gemv.h"
#include "cqil_internal.h"

namespace cqil {

constexpr int kU2 = 4;   // tiles in flight per strip when a wave walks two strips together
constexpr int kU1 = 8;   // tiles in flight when a wave walks one strip

// Combines the ksplit partial results of a unit.  Every wave of the workgroup calls this (it contains a
// barrier when ksplit > 1); afterwards the wave with ks == 0 holds the totals in y[].
template <int NY>
__device__ __forceinline__ void combine_ksplit(float (&y)[NY], int ksplit, int ul, int ks, float* red) {
    if (ksplit == 1) return;
    const int lane = threadIdx.x & 63;
    if (ks > 0 && lane < 16) {
#pragma unroll
        for (int n = 0; n < NY; ++n) red[((ul * ksplit + ks) * NY + n) * 16 + lane] = y[n];
    }
    __syncthreads();
    if (ks == 0 && lane < 16) {
        for (int s = 1; s < ksplit; ++s)
#pragma unroll
            for (int n = 0; n < NY; ++n) y[n] += red[((ul * ksplit + s) * NY + n) * 16 + lane];
    }
}
constexpr int kRedFloats = kWaves * 2 * 16;

// Second half of a norm prologue: xs[k] *= r * g[k] over the row, 16-byte chunks, one or two per thread for the
// LLaMA widths.  The first chunk of the gain row was requested by the caller before the barriers of its reduction
// (g0, chunk tid).  Ends with a barrier.
template <typename T>
__device__ __forceinline__ void scale_row_in_lds(float* xs, const T* g, const float (&g0)[elem<T>::kVec], float r,
                                                 int d_model) {
    constexpr int V = elem<T>::kVec;
    const int tid = threadIdx.x, n_chunks = d_model / V;
    for (int c = tid; c < n_chunks; c += kThreads) {
        float gv[V];
        if (c == tid) {
#pragma unroll
            for (int e = 0; e < V; ++e) gv[e] = g0[e];
        } else {
            elem<T>::unpack(load16(g + c * V), gv);
        }
#pragma unroll
        for (int e = 0; e < V; e += 4) {
            float4 t = *reinterpret_cast<float4*>(xs + c * V + e);
            t.x *= r * gv[e]; t.y *= r * gv[e + 1]; t.z *= r * gv[e + 2]; t.w *= r * gv[e + 3];
            *reinterpret_cast<float4*>(xs + c * V + e) = t;
        }
    }
    __syncthreads();
}  // [unit in workgroup][ks][NY <= 2][16], units * ksplit = waves

// ---------------------------------------------------------------------------------------------------------
// 1. RMSNorm + QKV projection + rotary embedding + KV append.  grid = (unit blocks, P); a unit is the pair of
//    strips holding rows (e, e + d_k/2), e = 16 tp .. 16 tp + 15, of one head of q, k or v.
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void qkv_rope_body(
    float* smem, int block, const T* __restrict__ x, const T* __restrict__ wqkv, const T* __restrict__ g_attn,
    const float2* __restrict__ rope, const int32_t* __restrict__ kv_len, T* __restrict__ kc, T* __restrict__ vc,
    float* __restrict__ q_out, int d_model, int n_heads, int d_k, int max_seq, int b_max, float eps, int ksplit) {
    constexpr int KB = tile<T>::KB, TE = tile<T>::kElems;
    float* xs = smem;             // d_model
    float* red = xs + d_model;    // kRedFloats
    float* scratch = red + kRedFloats;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int l = blockIdx.y;

    const int half = d_k >> 1;
    const int pairs_per_head = half / 16;
    const int units = 3 * n_heads * pairs_per_head;   // per layer
    const int uw = kWaves / ksplit;
    const int ul = w / ksplit, ks = w % ksplit;
    const int unit = block * uw + ul;
    const bool on = unit < units;
    const int tp = unit % pairs_per_head;
    const int hu = unit / pairs_per_head;
    const int h = hu % n_heads, m = hu / n_heads;  // m: 0,1,2 = q,k,v
    const int nkb = d_model / KB;
    const int per = (nkb + ksplit - 1) / ksplit;
    const int kb0 = min(ks * per, nkb), kb1 = min(kb0 + per, nkb);
    // the strips of the unit, and their first tiles on the way before the input vector is prepared
    const size_t strip_a = on ? ((size_t)(l * 3 + m) * d_model + (size_t)h * d_k + 16 * tp) / 16 : 0;
    const size_t strip_b = strip_a + half / 16;
    const T* strips[2] = {wqkv + (strip_a * nkb + kb0) * TE, wqkv + (strip_b * nkb + kb0) * TE};
    const int n_kb = on ? kb1 - kb0 : 0;
    uint4 wt[2][kU2];
    tile_strips_prefetch<T, 2, kU2>(strips, n_kb, wt);
    // the position and the rotation of the epilogue are requested now, not after the dot products
    const int pos = kv_len[0];
    float2 cs = make_float2(1.f, 0.f);
    if (on && ks == 0 && lane < 16 && m < 2 && pos >= 0 && pos < max_seq) cs = rope[(size_t)pos * half + 16 * tp + lane];

    // one statistic for the whole group: all P layers normalise the same x (Eq.3)
    constexpr int V = elem<T>::kVec;
    const int n_chunks = d_model / V;
    const T* g = g_attn + (size_t)l * d_model;
    float ss = 0.f;
    for (int c = tid; c < n_chunks; c += kThreads) {
        float v[V];
        elem<T>::unpack(load16(x + c * V), v);
#pragma unroll
        for (int e = 0; e < V; e += 4) {
            *reinterpret_cast<float4*>(xs + c * V + e) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
            ss += v[e] * v[e] + v[e + 1] * v[e + 1] + v[e + 2] * v[e + 2] + v[e + 3] * v[e + 3];
        }
    }
    float g0[V];  // requested before the reduction's barriers, used after them
    elem<T>::unpack(load16(g + min(tid, n_chunks - 1) * V), g0);
    ss = block_sum(ss, scratch);
    scale_row_in_lds<T>(xs, g, g0, 1.0f / sqrtf(ss / (float)d_model + eps), d_model);

    float y[2] = {0.f, 0.f};
    tile_strips_dot<T, 2, kU2>(strips, n_kb, xs + kb0 * KB, wt, y);
    combine_ksplit<2>(y, ksplit, ul, ks, red);

    if (on && ks == 0 && lane < 16 && pos >= 0 && pos < max_seq) {
        const int e = 16 * tp + lane;  // rotary pair (e, e + half)
        const float a = y[0], b = y[1];
        if (m == 2) {
            T* dst = vc + (((size_t)l * b_max * n_heads + h) * max_seq + pos) * d_k;
            elem<T>::store(dst + e, a);
            elem<T>::store(dst + e + half, b);
        } else {
            const float ra = a * cs.x - b * cs.y, rb = b * cs.x + a * cs.y;
            if (m == 0) {
                float* dst = q_out + (size_t)l * d_model + (size_t)h * d_k;
                dst[e] = ra;
                dst[e + half] = rb;
            } else {
                T* dst = kc + (((size_t)l * b_max * n_heads + h) * max_seq + pos) * d_k;
                elem<T>::store(dst + e, ra);
                elem<T>::store(dst + e + half, rb);
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void qkv_rope_kernel(
    const T* __restrict__ x, const T* __restrict__ wqkv, const T* __restrict__ g_attn, const float2* __restrict__ rope,
    const int32_t* __restrict__ kv_len, T* __restrict__ kc, T* __restrict__ vc, float* __restrict__ q_out,
    int d_model, int n_heads, int d_k, int max_seq, int b_max, float eps, int ksplit) {
    extern __shared__ float smem[];
    qkv_rope_body<T>(smem, blockIdx.x, x, wqkv, g_attn, rope, kv_len, kc, vc, q_out, d_model, n_heads, d_k, max_seq, b_max,
                     eps, ksplit);
}

// ---------------------------------------------------------------------------------------------------------
// 3. Output projection, per layer: a_l = Wo_l ctx_l.  grid = (unit blocks, P); a unit is one strip of 16 output
//    rows.  Wo is K-concatenated: the columns of layer l are the tiles l*d_model/KB .. of every strip.
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void oproj_body(float* smem, int l, const float* __restrict__ ctx, const T* __restrict__ wo,
                                           float* __restrict__ a, int P, int d_model, int ksplit) {
    constexpr int KB = tile<T>::KB, TE = tile<T>::kElems;
    float* xs = smem;
    float* red = xs + d_model;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int units = d_model / 16;
    const int uw = kWaves / ksplit;
    const int ul = w / ksplit, ks = w % ksplit;
    const int unit = blockIdx.x * uw + ul;
    const bool on = unit < units;
    const int nkb = d_model / KB;               // tiles of one layer
    const size_t strip_tiles = (size_t)P * nkb;  // tiles of a whole strip
    const int per = (nkb + ksplit - 1) / ksplit;
    const int kb0 = min(ks * per, nkb), kb1 = min(kb0 + per, nkb);
    const T* strips[1] = {wo + ((size_t)(on ? unit : 0) * strip_tiles + (size_t)l * nkb + kb0) * TE};
    const int n_kb = on ? kb1 - kb0 : 0;
    uint4 wt[1][kU1];
    tile_strips_prefetch<T, 1, kU1>(strips, n_kb, wt);  // weights on the way while the input goes to LDS

    const float* c = ctx + (size_t)l * d_model;
    for (int k = 4 * tid; k < d_model; k += 4 * kThreads)
        *reinterpret_cast<float4*>(xs + k) = *reinterpret_cast<const float4*>(c + k);
    __syncthreads();
    float y[1] = {0.f};
    tile_strips_dot<T, 1, kU1>(strips, n_kb, xs + kb0 * KB, wt, y);
    combine_ksplit<1>(y, ksplit, ul, ks, red);
    if (on && ks == 0 && lane < 16) a[(size_t)l * d_model + 16 * unit + lane] = y[0];
}

template <typename T>
__global__ __launch_bounds__(kThreads) void oproj_kernel(const float* __restrict__ ctx, const T* __restrict__ wo,
                                                          float* __restrict__ a, int P, int d_model, int ksplit) {
    extern __shared__ float smem[];
    oproj_body<T>(smem, blockIdx.y, ctx, wo, a, P, d_model, ksplit);
}

// ---------------------------------------------------------------------------------------------------------
// 4. Bypass window + FFN RMSNorm + gate/up projection + SwiGLU.  grid = (unit blocks, P); a unit is one packed
//    block: the strip of 16 gate rows and the strip of the matching 16 up rows.
//    h_l = x + sum_{j = max(0, l-d)}^{l} a_j   (Eq.4: own attention plus the d preceding layers' outputs)
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void gateup_body(float* smem, int block, const T* __restrict__ x, const float* __restrict__ a,
                                            const T* __restrict__ wgu, const T* __restrict__ g_ffn,
                                            float* __restrict__ u, int P, int bypass_d, int d_model, int d_ffn,
                                            float eps, int ksplit) {
    constexpr int KB = tile<T>::KB, TE = tile<T>::kElems;
    float* xs = smem;
    float* red = xs + d_model;
    float* scratch = red + kRedFloats;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int l = blockIdx.y;
    const int units = d_ffn / kGuBlock;
    const int uw = kWaves / ksplit;
    const int ul = w / ksplit, ks = w % ksplit;
    const int unit = block * uw + ul;
    const bool on = unit < units;
    const int nkb = d_model / KB;
    const int per = (nkb + ksplit - 1) / ksplit;
    const int kb0 = min(ks * per, nkb), kb1 = min(kb0 + per, nkb);
    const size_t strip_g = (size_t)l * 2 * d_ffn / 16 + 2 * (size_t)(on ? unit : 0);  // gate strip; the up strip follows
    const T* strips[2] = {wgu + (strip_g * nkb + kb0) * TE, wgu + ((strip_g + 1) * nkb + kb0) * TE};
    const int n_kb = on ? kb1 - kb0 : 0;
    uint4 wt[2][kU2];
    tile_strips_prefetch<T, 2, kU2>(strips, n_kb, wt);  // weights on the way while the input is formed

    const int jlo = bypass_d < 0 ? l + 1 : max(0, l - bypass_d);  // negative: Eq.5, the input is x alone
    constexpr int V = elem<T>::kVec;
    const int n_chunks = d_model / V;
    const T* g = g_ffn + (size_t)l * d_model;
    float ss = 0.f;
    for (int c = tid; c < n_chunks; c += kThreads) {
        float hv[V];
        elem<T>::unpack(load16(x + c * V), hv);
        for (int j = jlo; j <= l; ++j) {
            const float* ap = a + (size_t)j * d_model + c * V;
#pragma unroll
            for (int e = 0; e < V; e += 4) {
                const float4 t = *reinterpret_cast<const float4*>(ap + e);
                hv[e] += t.x; hv[e + 1] += t.y; hv[e + 2] += t.z; hv[e + 3] += t.w;
            }
        }
#pragma unroll
        for (int e = 0; e < V; e += 4) {
            *reinterpret_cast<float4*>(xs + c * V + e) = make_float4(hv[e], hv[e + 1], hv[e + 2], hv[e + 3]);
            ss += hv[e] * hv[e] + hv[e + 1] * hv[e + 1] + hv[e + 2] * hv[e + 2] + hv[e + 3] * hv[e + 3];
        }
    }
    float g0[V];  // requested before the reduction's barriers, used after them
    elem<T>::unpack(load16(g + min(tid, n_chunks - 1) * V), g0);
    ss = block_sum(ss, scratch);
    scale_row_in_lds<T>(xs, g, g0, 1.0f / sqrtf(ss / (float)d_model + eps), d_model);

    float y[2] = {0.f, 0.f};
    tile_strips_dot<T, 2, kU2>(strips, n_kb, xs + kb0 * KB, wt, y);
    combine_ksplit<2>(y, ksplit, ul, ks, red);
    if (on && ks == 0 && lane < 16)
        u[(size_t)l * d_ffn + unit * kGuBlock + lane] = y[0] / (1.0f + expf(-y[0])) * y[1];
}

template <typename T>
__global__ __launch_bounds__(kThreads) void gateup_kernel(const T* __restrict__ x, const float* __restrict__ a,
                                                           const T* __restrict__ wgu, const T* __restrict__ g_ffn,
                                                           float* __restrict__ u, int P, int bypass_d, int d_model,
                                                           int d_ffn, float eps, int ksplit) {
    extern __shared__ float smem[];
    gateup_body<T>(smem, blockIdx.x, x, a, wgu, g_ffn, u, P, bypass_d, d_model, d_ffn, eps, ksplit);
}

// Attention-FFN parallel form (App. A, Eq.5): every feed-forward module reads the shared input itself, so the QKV
// projection and the gate/up projection are two parts of ONE shared-input, N-concatenated product: one launch, one
// RMS statistic of x, two sets of gains (g_attn for the q/k/v rows, g_ffn for the gate/up rows).  Workgroups
// 0 .. q_blocks-1 of a layer take QKV units, the rest gate/up units.
template <typename T>
__global__ __launch_bounds__(kThreads) void qkv_gateup_kernel(
    const T* __restrict__ x, const T* __restrict__ wqkv, const T* __restrict__ g_attn, const float2* __restrict__ rope,
    const int32_t* __restrict__ kv_len, T* __restrict__ kc, T* __restrict__ vc, float* __restrict__ q_out,
    const T* __restrict__ wgu, const T* __restrict__ g_ffn, float* __restrict__ u, int P, int d_model, int n_heads,
    int d_k, int d_ffn, int max_seq, int b_max, float eps, int ksplit_q, int ksplit_g, int q_blocks) {
    extern __shared__ float smem[];
    if ((int)blockIdx.x < q_blocks)
        qkv_rope_body<T>(smem, blockIdx.x, x, wqkv, g_attn, rope, kv_len, kc, vc, q_out, d_model, n_heads, d_k, max_seq,
                         b_max, eps, ksplit_q);
    else
        gateup_body<T>(smem, (int)blockIdx.x - q_blocks, x, nullptr, wgu, g_ffn, u, P, CQIL_ATTN_FFN_PARALLEL, d_model,
                       d_ffn, eps, ksplit_g);
}

// ---------------------------------------------------------------------------------------------------------
// 5. Down projection over the K-concatenated Wdown [d_model][P*d_ffn (+ zero padding)]: the sum over the group's
//    layers in Eq.3 / Eq.4 is part of the dot product.  grid = (strip blocks, K slices); every slice writes its
//    partial sums, merge_kernel adds them in slice order (deterministic, no atomics).
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void down_body(float* smem, int slice, const float* __restrict__ u,
                                          const T* __restrict__ wdown, float* __restrict__ part, int K, int Kp,
                                          int d_model, int slice_len, int ksplit) {
    constexpr int KB = tile<T>::KB, TE = tile<T>::kElems;
    float* xs = smem;                 // slice_len
    float* red = xs + slice_len;      // kRedFloats
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int k0 = slice * slice_len;
    const int len = min(slice_len, Kp - k0);  // multiple of KB
    const int uw = kWaves / ksplit;
    const int ul = w / ksplit, ks = w % ksplit;
    const int unit = blockIdx.x * uw + ul;
    const bool on = unit < d_model / 16;
    const int nkb = len / KB;
    const int per = (nkb + ksplit - 1) / ksplit;
    const int kb0 = min(ks * per, nkb), kb1 = min(kb0 + per, nkb);
    const size_t strip_tiles = (size_t)Kp / KB;
    const T* strips[1] = {wdown + ((size_t)(on ? unit : 0) * strip_tiles + k0 / KB + kb0) * TE};
    const int n_kb = on ? kb1 - kb0 : 0;
    uint4 wt[1][kU1];
    tile_strips_prefetch<T, 1, kU1>(strips, n_kb, wt);  // weights on the way while the input goes to LDS

    for (int k = 4 * tid; k < len; k += 4 * kThreads) {  // len and K are multiples of 4
        const float4 t = (k0 + k < K) ? *reinterpret_cast<const float4*>(u + k0 + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        *reinterpret_cast<float4*>(xs + k) = t;
    }
    __syncthreads();
    float y[1] = {0.f};
    tile_strips_dot<T, 1, kU1>(strips, n_kb, xs + kb0 * KB, wt, y);
    combine_ksplit<1>(y, ksplit, ul, ks, red);
    if (on && ks == 0 && lane < 16) part[(size_t)slice * d_model + 16 * unit + lane] = y[0];
}

template <typename T>
__global__ __launch_bounds__(kThreads) void down_kernel(const float* __restrict__ u, const T* __restrict__ wdown,
                                                         float* __restrict__ part, int K, int Kp, int d_model,
                                                         int slice_len, int ksplit) {
    extern __shared__ float smem[];
    down_body<T>(smem, blockIdx.y, u, wdown, part, K, Kp, d_model, slice_len, ksplit);
}

// Eq.5's second contraction: without bypassing nothing needs a layer's attention output before its feed-forward
// output, so sum_l Wo_l ctx_l + sum_l Wdown_l u_l is ONE K-concatenated product [Wo_cat | Wdown_cat] [ctx; u]: one
// launch whose K slices are the P layers' segments of Wo (partial sums = the a_l, kept for the merge) followed by the
// slices of Wdown.  grid = (strip blocks, P + n_slices); the strip blocks of the two parts may differ in number
// (different k splits): a workgroup past its part's count has nothing to do.
template <typename T>
__global__ __launch_bounds__(kThreads) void oproj_down_kernel(const float* __restrict__ ctx, const T* __restrict__ wo,
                                                               float* __restrict__ a, const float* __restrict__ u,
                                                               const T* __restrict__ wdown, float* __restrict__ part,
                                                               int P, int K, int Kp, int d_model, int slice_len,
                                                               int ksplit_o, int ksplit_d) {
    extern __shared__ float smem[];
    if ((int)blockIdx.y < P)
        oproj_body<T>(smem, blockIdx.y, ctx, wo, a, P, d_model, ksplit_o);
    else
        down_body<T>(smem, (int)blockIdx.y - P, u, wdown, part, K, Kp, d_model, slice_len, ksplit_d);
}

// ---------------------------------------------------------------------------------------------------------
template <typename T>
static hipError_t decode_step_t(const StepArgs& s, hipStream_t st) {
    const cqil_dims& d = s.d;
    const int P = s.P, dm = d.d_model, f = d.d_ffn, dk = d.head_dim, nh = d.n_heads;
    const T* wqkv = (const T*)(s.packed + s.pl.wqkv);
    const T* wo = (const T*)(s.packed + s.pl.wo);
    const T* wgu = (const T*)(s.packed + s.pl.wgu);
    const T* wdown = (const T*)(s.packed + s.pl.wdown);
    const T* g_attn = (const T*)(s.packed + s.pl.g_attn);
    const T* g_ffn = (const T*)(s.packed + s.pl.g_ffn);
    const float2* rope = (const float2*)(s.packed + s.pl.rope);
    float* q = (float*)(s.ws + s.wl.q);
    float* ctx = (float*)(s.ws + s.wl.ctx);
    float* a = (float*)(s.ws + s.wl.a);
    float* u = (float*)(s.ws + s.wl.u);
    float* dpart = (float*)(s.ws + s.wl.down_part);
    const int bd = s.bypass_d >= P ? P - 1 : s.bypass_d;
    constexpr int KB = tile<T>::KB;
    const int K = P * f, Kp = (K + KB - 1) / KB * KB;
    // k splits, from measurements on 7B/13B/33B-shaped groups of 1, 2 and 4 layers: a kernel wants a certain number
    // of waves in total (units x P x split), so small groups split deeper; narrow models (short rows, where the
    // per-workgroup prologue weighs more) want fewer, fatter workgroups in the O, gate/up and down kernels.
    const bool narrow = dm <= 4096;
    auto split_for = [](long units, long want_waves) {
        int ks = 1;
        while (ks < 8 && units * ks < want_waves) ks *= 2;
        return ks;
    };
    const int t_q = g_tune.ksplit_qkv.load(), t_o = g_tune.ksplit_o.load(), t_g = g_tune.ksplit_gu.load(),
              t_d = g_tune.ksplit_d.load();
    const int ks_q = t_q ? t_q : split_for(3L * nh * (dk / 32) * P, 6144);
    const int ks_o = t_o ? t_o : ((narrow && P >= 4) ? 4 : 8);
    const int ks_g = t_g ? t_g : (narrow ? ((P == 2 || P == 3) ? 4 : 2) : split_for((long)(f / kGuBlock) * P, 16384));
    const size_t lds_x = ((size_t)dm + kRedFloats + 16) * sizeof(float);

    // optional per-kernel timing: event i is recorded before kernel i, the last event after the last kernel
#define CQIL_MARK(i) do { if (s.ev) (void)hipEventRecord(s.ev[i], st); } while (0)
    // Eq.5 (attention-FFN parallel form): three dependent phases instead of five -- QKV + gate/up in one shared-input
    // launch, attention, O + down in one K-concatenated launch -- then the merge.
    const bool fused = s.bypass_d < 0 && g_tune.eq5_fused.load() != 0;
    const int ks_d = t_d ? t_d : 8;
    CQIL_MARK(0);
    if (fused) {
        const int units_q = 3 * nh * (dk / 32), uw_q = kWaves / ks_q, q_blocks = (units_q + uw_q - 1) / uw_q;
        const int units_g = f / kGuBlock, uw_g = kWaves / ks_g, g_blocks = (units_g + uw_g - 1) / uw_g;
        hipLaunchKernelGGL(HIP_KERNEL_NAME(qkv_gateup_kernel<T>), dim3(q_blocks + g_blocks, P), dim3(kThreads), lds_x, st,
                           (const T*)s.x_in, wqkv, g_attn, rope, s.kv_len, (T*)s.kc, (T*)s.vc, q, wgu, g_ffn, u, P, dm, nh,
                           dk, f, d.max_seq, s.b_max, d.rms_eps, ks_q, ks_g, q_blocks);
    } else {
        const int units = 3 * nh * (dk / 32), uw = kWaves / ks_q;
        hipLaunchKernelGGL(HIP_KERNEL_NAME(qkv_rope_kernel<T>), dim3((units + uw - 1) / uw, P), dim3(kThreads), lds_x, st,
                           (const T*)s.x_in, wqkv, g_attn, rope, s.kv_len, (T*)s.kc, (T*)s.vc, q, dm, nh, dk,
                           d.max_seq, s.b_max, d.rms_eps, ks_q);
    }
    CQIL_MARK(1);
    const int lps = dk * (int)sizeof(T) / 16;
#define CQIL_ATTN(LPS)                                                                                               \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(attn_decode_kernel<T, float, LPS, kAttnWaves>), dim3(P * nh), dim3(kAttnThreads), 0, \
                       st, (const float*)q, (size_t)dm, (size_t)dm, (const T*)s.kc, (const T*)s.vc, s.kv_len, ctx, 1, 1, nh,    \
                       d.max_seq, s.b_max)
    switch (lps) {
        case 4: CQIL_ATTN(4); break;
        case 8: CQIL_ATTN(8); break;
        case 16: CQIL_ATTN(16); break;
        case 32: CQIL_ATTN(32); break;
        case 64: CQIL_ATTN(64); break;
        default: return hipErrorInvalidValue;
    }
#undef CQIL_ATTN
    CQIL_MARK(2);
    if (fused) {
        const int units = dm / 16, uw_o = kWaves / ks_o, uw_d = kWaves / ks_d;
        const int blocks = max((units + uw_o - 1) / uw_o, (units + uw_d - 1) / uw_d);
        const size_t lds = ((size_t)max(dm, s.wl.down_slice) + kRedFloats + 16) * sizeof(float);
        hipLaunchKernelGGL(HIP_KERNEL_NAME(oproj_down_kernel<T>), dim3(blocks, P + s.wl.n_slices), dim3(kThreads), lds, st,
                           ctx, wo, a, u, wdown, dpart, P, K, Kp, dm, s.wl.down_slice, ks_o, ks_d);
        CQIL_MARK(3);
        CQIL_MARK(4);
    } else {
        {
            const int units = dm / 16, uw = kWaves / ks_o;
            hipLaunchKernelGGL(HIP_KERNEL_NAME(oproj_kernel<T>), dim3((units + uw - 1) / uw, P), dim3(kThreads), lds_x, st,
                               ctx, wo, a, P, dm, ks_o);
        }
        CQIL_MARK(3);
        {
            const int units = f / kGuBlock, uw = kWaves / ks_g;
            hipLaunchKernelGGL(HIP_KERNEL_NAME(gateup_kernel<T>), dim3((units + uw - 1) / uw, P), dim3(kThreads), lds_x, st,
                               (const T*)s.x_in, a, wgu, g_ffn, u, P, bd, dm, f, d.rms_eps, ks_g);
        }
        CQIL_MARK(4);
        {
            const int units = dm / 16, uw = kWaves / ks_d;
            hipLaunchKernelGGL(HIP_KERNEL_NAME(down_kernel<T>), dim3((units + uw - 1) / uw, s.wl.n_slices), dim3(kThreads),
                               ((size_t)s.wl.down_slice + kRedFloats) * sizeof(float), st, u, wdown, dpart, K, Kp, dm,
                               s.wl.down_slice, ks_d);
        }
    }
    CQIL_MARK(5);
    hipLaunchKernelGGL(HIP_KERNEL_NAME(merge_kernel<T>), dim3((dm + 63) / 64), dim3(64 * kMergeY), 0, st,
                       (const T*)s.x_res, a, dpart, (T*)s.x_out, s.kv_len, s.advance, P, s.wl.n_slices, dm, 1, 1);
    CQIL_MARK(6);
#undef CQIL_MARK
    return hipGetLastError();
}

hipError_t launch_decode_step(const StepArgs& s, hipStream_t st) {
    return s.d.dtype == CQIL_BF16 ? decode_step_t<bf16_t>(s, st) : decode_step_t<float>(s, st);
}

}  // namespace cqil
