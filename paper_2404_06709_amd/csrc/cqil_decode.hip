// Decode step of one CQIL group for a single new token (B*T == 1): five bandwidth-bound kernels and a merge.
//
//   1 qkv_rope   shared-input projection of all P layers (Eq.2's xW^Q, xW^K, xW^V applied to the one x_G of
//                Eq.3), fused with the attention RMSNorm (one statistic for the whole group, P gains), the
//                rotary embedding and the KV-cache append
//   2 attn       softmax(QK^T/sqrt(d_k))V over the P independent caches, split along the cache length
//   3 oproj      per-layer Concat(heads)W^O
//   4 gateup     forms the P feed-forward inputs h_i = x + a_i + bypass window (Eq.4), their RMSNorm, the
//                gate/up projections and SwiGLU
//   5 down       one contraction over the K-concatenated Wdown: sum_i FFN_i, split along K
//   6 merge      x_out = x + sum_i a_i + sum of the K slices (Eq.3 / Eq.4)
//
// Every projection is a matrix-vector product streamed once from HBM: a wave owns four rows at a time, each
// lane reads 16 contiguous bytes of each row per step, the input vector sits in LDS as fp32.
#include "cqil_dev.h"
#include "cqil_attn.h"
#include "cqil_gemv.h"
#include "cqil_internal.h"

namespace cqil {

// ---------------------------------------------------------------------------------------------------------
// 1. RMSNorm + QKV projection + rotary embedding + KV append.  One workgroup per (layer, q|k|v, head).
// ---------------------------------------------------------------------------------------------------------
template <typename T, int PIPE>
__global__ __launch_bounds__(kThreads) void qkv_rope_kernel(
    const T* __restrict__ x, const T* __restrict__ wqkv, const T* __restrict__ g_attn, const float2* __restrict__ rope,
    const int32_t* __restrict__ kv_len, T* __restrict__ kc, T* __restrict__ vc, float* __restrict__ q_out,
    int d_model, int n_heads, int d_k, int max_seq, int b_max, float eps, int parts) {
    extern __shared__ float smem[];
    constexpr int V = elem<T>::kVec;
    float* xs = smem;                        // xs_words(d_model)
    float* y = xs + xs_words(d_model);       // d_k
    float* scratch = y + d_k;                // 16
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int unit = blockIdx.x / parts, part = blockIdx.x % parts;  // a head may be split over several workgroups
    const int h = unit % n_heads;
    const int lm = unit / n_heads;  // l*3 + m
    const int l = lm / 3, m = lm % 3;

    // one statistic for the whole group: all P layers normalise the same x (Eq.3)
    float ss = 0.f;
    for (int k = tid; k < d_model; k += kThreads) {
        const float v = elem<T>::load(x + k);
        ss += v * v;
    }
    ss = block_sum(ss, scratch);
    const float r = 1.0f / sqrtf(ss / (float)d_model + eps);
    const T* g = g_attn + (size_t)l * d_model;
    for (int k = tid; k < d_model; k += kThreads)
        xs[xs_index<V>(k)] = elem<T>::load(x + k) * r * elem<T>::load(g + k);
    __syncthreads();

    // rows of this head; a wave takes the two rows of a rotary pair together: (e, e + d_k/2)
    const int half = d_k >> 1;
    const T* wbase = wqkv + ((size_t)lm * d_model + (size_t)h * d_k) * d_model;
    const int gp = half / 2 / parts;  // groups of two rotary pairs handled by this workgroup
    stream_rows<T, PIPE>(
        part * gp + w, (part + 1) * gp, kWaves, d_model, xs,
        [&](int g, const T* (&r)[4]) {
            const int e0 = 2 * g;
            r[0] = wbase + (size_t)e0 * d_model;
            r[1] = wbase + (size_t)(e0 + 1) * d_model;
            r[2] = wbase + (size_t)(e0 + half) * d_model;
            r[3] = wbase + (size_t)(e0 + 1 + half) * d_model;
        },
        [&](int g, const float (&s)[4]) {
            const int e0 = 2 * g;
            if (lane == 0) { y[e0] = s[0]; y[e0 + 1] = s[1]; y[e0 + half] = s[2]; y[e0 + 1 + half] = s[3]; }
        });
    __syncthreads();

    const int pos = kv_len[0];
    const int i = part * 2 * gp + tid;  // rotary pair (i, i + half)
    if (tid < 2 * gp && pos >= 0 && pos < max_seq) {
        const float a = y[i], b = y[i + half];
        if (m == 2) {
            T* dst = vc + (((size_t)l * b_max * n_heads + h) * max_seq + pos) * d_k;
            elem<T>::store(dst + i, a);
            elem<T>::store(dst + i + half, b);
        } else {
            const float2 cs = rope[(size_t)pos * half + i];
            const float ra = a * cs.x - b * cs.y, rb = b * cs.x + a * cs.y;
            if (m == 0) {
                float* dst = q_out + (size_t)l * d_model + (size_t)h * d_k;
                dst[i] = ra;
                dst[i + half] = rb;
            } else {
                T* dst = kc + (((size_t)l * b_max * n_heads + h) * max_seq + pos) * d_k;
                elem<T>::store(dst + i, ra);
                elem<T>::store(dst + i + half, rb);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// 2. Decode attention over P independent caches.  One workgroup of 16 waves per (layer, sequence, head): every
//    wave walks the cache in strides, four slot steps (K and V loads of all four in flight) per iteration, with a
//    running maximum / sum / context (online softmax); the 16 partial results are merged through LDS.
//    LPS = lanes that share one cache slot = head_dim * sizeof(T) / 16.
// ---------------------------------------------------------------------------------------------------------
// (kernel in cqil_attn.h)

// ---------------------------------------------------------------------------------------------------------
// 3. Output projection, per layer: a_l = Wo_l ctx_l.  grid = (row blocks, P).  Wo is K-concatenated:
//    packed row o holds the P layers' rows side by side, layer l's segment starts at l*d_model.
// ---------------------------------------------------------------------------------------------------------
template <typename T, int PIPE>
__global__ __launch_bounds__(kThreads) void oproj_kernel(const float* __restrict__ ctx, const T* __restrict__ wo,
                                                          float* __restrict__ a, int P, int d_model, int rows_per_wg) {
    extern __shared__ float smem[];
    constexpr int V = elem<T>::kVec;
    float* xs = smem;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int l = blockIdx.y;
    const float* c = ctx + (size_t)l * d_model;
    for (int k = tid; k < d_model; k += kThreads) xs[xs_index<V>(k)] = c[k];
    __syncthreads();
    const int row0 = blockIdx.x * rows_per_wg;
    const int row1 = min(row0 + rows_per_wg, d_model);
    const size_t ld = (size_t)P * d_model;
    stream_rows<T, PIPE>(
        w, (row1 - row0) / 4, kWaves, d_model, xs,
        [&](int g, const T* (&r)[4]) {
            const T* p = wo + (size_t)(row0 + 4 * g) * ld + (size_t)l * d_model;
            r[0] = p; r[1] = p + ld; r[2] = p + 2 * ld; r[3] = p + 3 * ld;
        },
        [&](int g, const float (&s)[4]) {
            if (lane == 0)
                *reinterpret_cast<float4*>(a + (size_t)l * d_model + row0 + 4 * g) = make_float4(s[0], s[1], s[2], s[3]);
        });
}

// ---------------------------------------------------------------------------------------------------------
// 4. Bypass window + FFN RMSNorm + gate/up projection + SwiGLU.  grid = (blocks of j, P).
//    h_l = x + sum_{j = max(0, l-d)}^{l} a_j   (Eq.4: own attention plus the d preceding layers' outputs)
// ---------------------------------------------------------------------------------------------------------
template <typename T, int PIPE>
__global__ __launch_bounds__(kThreads) void gateup_kernel(const T* __restrict__ x, const float* __restrict__ a,
                                                           const T* __restrict__ wgu, const T* __restrict__ g_ffn,
                                                           float* __restrict__ u, int P, int bypass_d, int d_model,
                                                           int d_ffn, int j_per_wg, float eps) {
    extern __shared__ float smem[];
    constexpr int V = elem<T>::kVec;
    float* xs = smem;
    float* scratch = xs + xs_words(d_model);
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int l = blockIdx.y;
    const int jlo = max(0, l - bypass_d);
    float ss = 0.f;
    for (int k = tid; k < d_model; k += kThreads) {
        float hv = elem<T>::load(x + k);
        for (int j = jlo; j <= l; ++j) hv += a[(size_t)j * d_model + k];
        xs[xs_index<V>(k)] = hv;
        ss += hv * hv;
    }
    ss = block_sum(ss, scratch);
    const float r = 1.0f / sqrtf(ss / (float)d_model + eps);
    const T* g = g_ffn + (size_t)l * d_model;
    for (int k = tid; k < d_model; k += kThreads) xs[xs_index<V>(k)] *= r * elem<T>::load(g + k);
    __syncthreads();

    const int j0 = blockIdx.x * j_per_wg;
    const int j1 = min(j0 + j_per_wg, d_ffn);
    const T* wl = wgu + (size_t)l * 2 * d_ffn * d_model;
    stream_rows<T, PIPE>(
        w, (j1 - j0) / 2, kWaves, d_model, xs,
        [&](int g, const T* (&r)[4]) {
            // packed row of gate j: block (j/16) of 32 rows, gate rows first, then the up rows
            const int j = j0 + 2 * g;
            const T* rg = wl + ((size_t)(j / kGuBlock) * 2 * kGuBlock + (j % kGuBlock)) * d_model;
            const T* ru = rg + (size_t)kGuBlock * d_model;
            r[0] = rg; r[1] = rg + d_model; r[2] = ru; r[3] = ru + d_model;
        },
        [&](int g, const float (&s)[4]) {
            if (lane == 0) {
                const int j = j0 + 2 * g;
                const float u0 = s[0] / (1.0f + expf(-s[0])) * s[2];
                const float u1 = s[1] / (1.0f + expf(-s[1])) * s[3];
                *reinterpret_cast<float2*>(u + (size_t)l * d_ffn + j) = make_float2(u0, u1);
            }
        });
}

// ---------------------------------------------------------------------------------------------------------
// 5. Down projection over the K-concatenated Wdown [d_model][P*d_ffn]: the sum over the group's layers in
//    Eq.3 / Eq.4 is part of the dot product.  grid = (row blocks, K slices); every slice writes its partial
//    sums, the merge kernel below adds them in slice order (deterministic, no atomics).
// ---------------------------------------------------------------------------------------------------------
template <typename T, int PIPE>
__global__ __launch_bounds__(kThreads) void down_kernel(const float* __restrict__ u, const T* __restrict__ wdown,
                                                         float* __restrict__ part, int P, int d_model, int d_ffn,
                                                         int rows_per_wg, int slice_len) {
    extern __shared__ float smem[];
    constexpr int V = elem<T>::kVec;
    float* xs = smem;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int K = P * d_ffn;
    const int slice = blockIdx.y;
    const int k0 = slice * slice_len;
    const int len = min(slice_len, K - k0);
    for (int k = tid; k < len; k += kThreads) xs[xs_index<V>(k)] = u[k0 + k];
    __syncthreads();
    const int row0 = blockIdx.x * rows_per_wg;
    const int row1 = min(row0 + rows_per_wg, d_model);
    float* mypart = part + (size_t)slice * d_model;
    stream_rows<T, PIPE>(
        w, (row1 - row0) / 4, kWaves, len, xs,
        [&](int g, const T* (&r)[4]) {
            const T* p = wdown + (size_t)(row0 + 4 * g) * K + k0;
            r[0] = p; r[1] = p + K; r[2] = p + 2 * (size_t)K; r[3] = p + 3 * (size_t)K;
        },
        [&](int g, const float (&s)[4]) {
            if (lane == 0) *reinterpret_cast<float4*>(mypart + row0 + 4 * g) = make_float4(s[0], s[1], s[2], s[3]);
        });
}

// 6. Merge of Eq.3 / Eq.4: merge_kernel in cqil_attn.h

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
    const int xw = (dm + 511) & ~511;
    // launch shapes: measured on 7B/13B/33B-shaped groups; the O projection wants at least ~400 workgroups,
    // the gate/up kernel ~0.7-1 MB of weights per workgroup
    int rows_o = g_tune.rows_o, j_per = g_tune.j_per;
    const int rows_d = g_tune.rows_d;
    if (rows_o == 0) {
        rows_o = 64;
        while (rows_o > 16 && ((dm + rows_o - 1) / rows_o) * P < 400) rows_o >>= 1;
    }
    if (j_per == 0) j_per = dm <= 4096 ? 64 : 32;
    const int pipe = g_tune.pipeline;
    int parts = g_tune.qkv_parts;
    while (parts > 1 && (dk / 4) % parts) parts >>= 1;  // whole groups of two rotary pairs per workgroup

    // optional per-kernel timing: event i is recorded before kernel i, the last event after the last kernel
#define CQIL_MARK(i) do { if (s.ev) (void)hipEventRecord(s.ev[i], st); } while (0)
    CQIL_MARK(0);
#define CQIL_QKV(PIPE)                                                                                               \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(qkv_rope_kernel<T, PIPE>), dim3(P * 3 * nh * parts), dim3(kThreads),          \
                       (xw + dk + 16) * sizeof(float), st, (const T*)s.x_in, wqkv, g_attn, rope, s.kv_len, (T*)s.kc, \
                       (T*)s.vc, q, dm, nh, dk, d.max_seq, s.b_max, d.rms_eps, parts)
    switch (pipe) { case 1: CQIL_QKV(1); break; case 2: CQIL_QKV(2); break; case 3: CQIL_QKV(3); break; default: CQIL_QKV(0); }
#undef CQIL_QKV
    CQIL_MARK(1);
    const int lps = dk * (int)sizeof(T) / 16;
#define CQIL_ATTN(LPS)                                                                                               \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(attn_decode_kernel<T, LPS>), dim3(P * nh), dim3(kAttnThreads), 0, st, q,      \
                       (const T*)s.kc, (const T*)s.vc, s.kv_len, ctx, 1, 1, nh, d.max_seq, s.b_max)
    switch (lps) {
        case 4: CQIL_ATTN(4); break;
        case 8: CQIL_ATTN(8); break;
        case 16: CQIL_ATTN(16); break;
        case 32: CQIL_ATTN(32); break;
        default: return hipErrorInvalidValue;
    }
#undef CQIL_ATTN
    CQIL_MARK(2);
#define CQIL_OPROJ(PIPE)                                                                                             \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(oproj_kernel<T, PIPE>), dim3((dm + rows_o - 1) / rows_o, P), dim3(kThreads),  \
                       xw * sizeof(float), st, ctx, wo, a, P, dm, rows_o)
    switch (pipe) { case 1: CQIL_OPROJ(1); break; case 2: CQIL_OPROJ(2); break; case 3: CQIL_OPROJ(3); break; default: CQIL_OPROJ(0); }
#undef CQIL_OPROJ
    CQIL_MARK(3);
#define CQIL_GATEUP(PIPE)                                                                                            \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(gateup_kernel<T, PIPE>), dim3((f + j_per - 1) / j_per, P), dim3(kThreads),    \
                       (xw + 16) * sizeof(float), st, (const T*)s.x_in, a, wgu, g_ffn, u, P, bd, dm, f, j_per,       \
                       d.rms_eps)
    switch (pipe) { case 1: CQIL_GATEUP(1); break; case 2: CQIL_GATEUP(2); break; case 3: CQIL_GATEUP(3); break; default: CQIL_GATEUP(0); }
#undef CQIL_GATEUP
    CQIL_MARK(4);
#define CQIL_DOWN(PIPE)                                                                                              \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(down_kernel<T, PIPE>), dim3((dm + rows_d - 1) / rows_d, s.wl.n_slices),       \
                       dim3(kThreads), ((s.wl.down_slice + 511) & ~511) * sizeof(float), st, u, wdown, dpart, P, dm, \
                       f, rows_d, s.wl.down_slice)
    switch (pipe) { case 1: CQIL_DOWN(1); break; case 2: CQIL_DOWN(2); break; case 3: CQIL_DOWN(3); break; default: CQIL_DOWN(0); }
#undef CQIL_DOWN
    CQIL_MARK(5);
    hipLaunchKernelGGL(HIP_KERNEL_NAME(merge_kernel<T>), dim3((dm + 255) / 256, 1), dim3(256), 0, st, (const T*)s.x_in,
                       a, dpart, (T*)s.x_out, s.kv_len, s.advance, P, s.wl.n_slices, 1, dm, 1, 1);
    CQIL_MARK(6);
#undef CQIL_MARK
    return hipGetLastError();
}

hipError_t launch_decode_step(const StepArgs& s, hipStream_t st) {
    return s.d.dtype == CQIL_BF16 ? decode_step_t<bf16_t>(s, st) : decode_step_t<float>(s, st);
}

}  // namespace cqil
