// Decode step of one CQIL group for a single new token (B*T == 1): five bandwidth-bound kernels.
//
//   1 qkv_rope   shared-input projection of all P layers (Eq.2's xW^Q, xW^K, xW^V applied to the one x_G of
//                Eq.3), fused with the attention RMSNorm (one statistic for the whole group, P gains), the
//                rotary embedding and the KV-cache append
//   2 attn       softmax(QK^T/sqrt(d_k))V over the P independent caches, split along the cache length
//   3 oproj      per-layer Concat(heads)W^O
//   4 gateup     forms the P feed-forward inputs h_i = x + a_i + bypass window (Eq.4), their RMSNorm, the
//                gate/up projections and SwiGLU
//   5 down       one contraction over the K-concatenated Wdown: sum_i FFN_i, plus x + sum_i a_i (Eq.3/Eq.4)
//
// Every projection is a matrix-vector product streamed once from HBM: a wave owns four rows at a time, each
// lane reads 16 contiguous bytes of each row per step, the input vector sits in LDS as fp32.
#include "cqil_dev.h"
#include "cqil_gemv.h"
#include "cqil_internal.h"

namespace cqil {

// ---------------------------------------------------------------------------------------------------------
// 1. RMSNorm + QKV projection + rotary embedding + KV append.  One workgroup per (layer, q|k|v, head).
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void qkv_rope_kernel(
    const T* __restrict__ x, const T* __restrict__ wqkv, const T* __restrict__ g_attn, const float2* __restrict__ rope,
    const int32_t* __restrict__ kv_len, T* __restrict__ kc, T* __restrict__ vc, float* __restrict__ q_out,
    int32_t* __restrict__ counters, int n_counters, int d_model, int n_heads, int d_k, int max_seq, int b_max,
    float eps) {
    extern __shared__ float smem[];
    constexpr int V = elem<T>::kVec;
    float* xs = smem;                        // xs_words(d_model)
    float* y = xs + xs_words(d_model);       // d_k
    float* scratch = y + d_k;                // 16
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int unit = blockIdx.x;
    const int h = unit % n_heads;
    const int lm = unit / n_heads;  // l*3 + m
    const int l = lm / 3, m = lm % 3;

    if (unit == 0)
        for (int i = tid; i < n_counters; i += kThreads) counters[i] = 0;

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
    for (int e0 = 2 * w; e0 < half; e0 += 2 * kWaves) {
        float s[4];
        dot4<T>(wbase + (size_t)e0 * d_model, wbase + (size_t)(e0 + 1) * d_model,
                wbase + (size_t)(e0 + half) * d_model, wbase + (size_t)(e0 + 1 + half) * d_model, xs, d_model, s);
        if (lane == 0) { y[e0] = s[0]; y[e0 + 1] = s[1]; y[e0 + half] = s[2]; y[e0 + 1 + half] = s[3]; }
    }
    __syncthreads();

    const int pos = kv_len[0];
    if (tid < half && pos >= 0 && pos < max_seq) {
        const float a = y[tid], b = y[tid + half];
        if (m == 2) {
            T* dst = vc + (((size_t)l * b_max * n_heads + h) * max_seq + pos) * d_k;
            elem<T>::store(dst + tid, a);
            elem<T>::store(dst + tid + half, b);
        } else {
            const float2 cs = rope[(size_t)pos * half + tid];
            const float ra = a * cs.x - b * cs.y, rb = b * cs.x + a * cs.y;
            if (m == 0) {
                float* dst = q_out + (size_t)l * d_model + (size_t)h * d_k;
                dst[tid] = ra;
                dst[tid + half] = rb;
            } else {
                T* dst = kc + (((size_t)l * b_max * n_heads + h) * max_seq + pos) * d_k;
                elem<T>::store(dst + tid, ra);
                elem<T>::store(dst + tid + half, rb);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// 2. Decode attention over P independent caches, split along the cache length.
//    grid = (P*B*n_heads, n_chunks).  Each workgroup reduces kAttnChunk slots to (max, sum, context); the
//    last workgroup of a (layer, sequence, head) to arrive merges the chunks in chunk order.
//    LPS = lanes that share one cache slot = head_dim * sizeof(T) / 16.
// ---------------------------------------------------------------------------------------------------------
template <typename T, int LPS>
__global__ __launch_bounds__(kThreads) void attn_decode_kernel(
    const float* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc,
    const int32_t* __restrict__ kv_len, float* __restrict__ part, int32_t* __restrict__ counters,
    float* __restrict__ ctx, int B, int n_heads, int max_seq, int b_max, int n_chunks) {
    constexpr int V = elem<T>::kVec;
    constexpr int DK = LPS * V;
    constexpr int SPW = kWave / LPS;                      // slots per wave step
    constexpr int NI = kAttnChunk / kWaves / SPW;         // steps per wave
    __shared__ float red[2 * kWaves];
    __shared__ float accs[kWaves][DK];
    __shared__ int s_last;

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int sub = lane % LPS, sg = lane / LPS;
    const int unit = blockIdx.x, chunk = blockIdx.y;
    const int h = unit % n_heads;
    const int lb = unit / n_heads;
    const int b = lb % B, l = lb / B;
    int S = kv_len[b] + 1;  // slots to attend, including the token appended by the previous kernel
    if (S > max_seq) S = max_seq;
    if (S < 1) return;
    const int n_valid = (S + kAttnChunk - 1) / kAttnChunk;
    if (chunk >= n_valid) return;

    const size_t d_model = (size_t)n_heads * DK;
    const float scale = 1.0f / sqrtf((float)DK);
    float qv[V];
    {
        const float* qp = q + ((size_t)l * B + b) * d_model + (size_t)h * DK + sub * V;
#pragma unroll
        for (int j = 0; j < V; ++j) qv[j] = qp[j] * scale;
    }
    const size_t head_off = (((size_t)l * b_max + b) * n_heads + h) * (size_t)max_seq * DK;
    const T* kb = kc + head_off;
    const T* vb = vc + head_off;
    const int s0 = chunk * kAttnChunk + w * (kAttnChunk / kWaves) + sg;

    float sc[NI];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int s = s0 + i * SPW;
        float dot = 0.f;
        if (s < S) {
            float f[V];
            elem<T>::unpack(load16(kb + (size_t)s * DK + sub * V), f);
#pragma unroll
            for (int j = 0; j < V; ++j) dot = fmaf(f[j], qv[j], dot);
        }
#pragma unroll
        for (int off = LPS / 2; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, kWave);
        sc[i] = (s < S) ? dot : -INFINITY;
        mx = fmaxf(mx, sc[i]);
    }
    mx = wave_max(mx);
    if (lane == 0) red[w] = mx;
    __syncthreads();
    mx = red[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) mx = fmaxf(mx, red[i]);  // finite: slot chunk*kAttnChunk < S

    float acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = 0.f;
    float lsum = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int s = s0 + i * SPW;
        if (s < S) {
            const float p = expf(sc[i] - mx);
            lsum += p;
            float f[V];
            elem<T>::unpack(load16(vb + (size_t)s * DK + sub * V), f);
#pragma unroll
            for (int j = 0; j < V; ++j) acc[j] = fmaf(p, f[j], acc[j]);
        }
    }
    // combine the SPW slot groups of the wave
#pragma unroll
    for (int off = LPS; off < kWave; off <<= 1) {
        lsum += __shfl_xor(lsum, off, kWave);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] += __shfl_xor(acc[j], off, kWave);
    }
    if (sg == 0) {
#pragma unroll
        for (int j = 0; j < V; ++j) accs[w][sub * V + j] = acc[j];
    }
    if (lane == 0) red[kWaves + w] = lsum;
    __syncthreads();
    float ltot = 0.f;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) ltot += red[kWaves + i];

    float* ctx_out = ctx + ((size_t)l * B + b) * d_model + (size_t)h * DK;
    if (n_valid == 1) {
        if (tid < DK) {
            float c = 0.f;
#pragma unroll
            for (int i = 0; i < kWaves; ++i) c += accs[i][tid];
            ctx_out[tid] = c / ltot;
        }
        return;
    }
    float* mypart = part + ((size_t)unit * n_chunks + chunk) * (DK + 2);
    if (tid < DK) {
        float c = 0.f;
#pragma unroll
        for (int i = 0; i < kWaves; ++i) c += accs[i][tid];
        mypart[2 + tid] = c;
    }
    if (tid == 0) { mypart[0] = mx; mypart[1] = ltot; }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int ticket = __hip_atomic_fetch_add(&counters[unit], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (ticket == n_valid - 1);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (tid < DK) {
        const float* up = part + (size_t)unit * n_chunks * (DK + 2);
        float M = -INFINITY;
        for (int c = 0; c < n_valid; ++c)
            M = fmaxf(M, __hip_atomic_load(up + (size_t)c * (DK + 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        float Lsum = 0.f, cacc = 0.f;
        for (int c = 0; c < n_valid; ++c) {
            const float* pc = up + (size_t)c * (DK + 2);
            const float e = expf(__hip_atomic_load(pc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - M);
            Lsum += e * __hip_atomic_load(pc + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            cacc += e * __hip_atomic_load(pc + 2 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        ctx_out[tid] = cacc / Lsum;
    }
    if (tid == 0) counters[unit] = 0;
}

// ---------------------------------------------------------------------------------------------------------
// 3. Output projection, per layer: a_l = Wo_l ctx_l.  grid = (row blocks, P).  Wo is K-concatenated:
//    packed row o holds the P layers' rows side by side, layer l's segment starts at l*d_model.
// ---------------------------------------------------------------------------------------------------------
template <typename T>
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
    for (int o = row0 + 4 * w; o < row1; o += 4 * kWaves) {
        const T* r = wo + (size_t)o * ld + (size_t)l * d_model;
        float s[4];
        dot4<T>(r, r + ld, r + 2 * ld, r + 3 * ld, xs, d_model, s);
        if (lane == 0) {
            float4 v = make_float4(s[0], s[1], s[2], s[3]);
            *reinterpret_cast<float4*>(a + (size_t)l * d_model + o) = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// 4. Bypass window + FFN RMSNorm + gate/up projection + SwiGLU.  grid = (blocks of j, P).
//    h_l = x + sum_{j = max(0, l-d)}^{l} a_j   (Eq.4: own attention plus the d preceding layers' outputs)
// ---------------------------------------------------------------------------------------------------------
template <typename T>
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
    for (int j = j0 + 2 * w; j < j1; j += 2 * kWaves) {
        // packed row of gate j: block (j/16) of 32 rows, gate rows first, then the up rows
        const T* rg = wl + ((size_t)(j / kGuBlock) * 2 * kGuBlock + (j % kGuBlock)) * d_model;
        const T* ru = rg + (size_t)kGuBlock * d_model;
        float s[4];
        dot4<T>(rg, rg + d_model, ru, ru + d_model, xs, d_model, s);
        if (lane == 0) {
            const float u0 = s[0] / (1.0f + expf(-s[0])) * s[2];
            const float u1 = s[1] / (1.0f + expf(-s[1])) * s[3];
            *reinterpret_cast<float2*>(u + (size_t)l * d_ffn + j) = make_float2(u0, u1);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// 5. Down projection over the K-concatenated Wdown [d_model][P*d_ffn] with the merge of Eq.3 / Eq.4:
//    x_out = x + sum_i a_i + Wdown_cat u_cat.   grid = (row blocks, K slices).  With more than one slice the
//    last workgroup of a row block to arrive adds the slices in slice order (deterministic).
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void down_kernel(const T* __restrict__ x, const float* __restrict__ a,
                                                         const float* __restrict__ u, const T* __restrict__ wdown,
                                                         float* __restrict__ part, int32_t* __restrict__ counters,
                                                         T* __restrict__ x_out, int32_t* __restrict__ kv_len, int advance,
                                                         int P, int d_model, int d_ffn, int rows_per_wg, int slice_len) {
    extern __shared__ float smem[];
    constexpr int V = elem<T>::kVec;
    __shared__ int s_last;
    float* xs = smem;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int K = P * d_ffn;
    const int slice = blockIdx.y, n_slices = gridDim.y;
    const int k0 = slice * slice_len;
    const int len = min(slice_len, K - k0);
    for (int k = tid; k < len; k += kThreads) xs[xs_index<V>(k)] = u[k0 + k];
    __syncthreads();
    const int row0 = blockIdx.x * rows_per_wg;
    const int row1 = min(row0 + rows_per_wg, d_model);
    float* mypart = part + (size_t)slice * d_model;
    for (int o = row0 + 4 * w; o < row1; o += 4 * kWaves) {
        const T* r = wdown + (size_t)o * K + k0;
        float s[4];
        dot4<T>(r, r + K, r + 2 * (size_t)K, r + 3 * (size_t)K, xs, len, s);
        if (lane == 0) *reinterpret_cast<float4*>(mypart + o) = make_float4(s[0], s[1], s[2], s[3]);
    }
    if (advance && blockIdx.x == 0 && slice == 0 && tid == 0) kv_len[0] += 1;

    if (n_slices > 1) {
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            const int ticket =
                __hip_atomic_fetch_add(&counters[blockIdx.x], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (ticket == n_slices - 1);
        }
        __syncthreads();
        if (!s_last) return;
        __threadfence();
    } else {
        __syncthreads();
    }
    for (int o = row0 + tid; o < row1; o += kThreads) {
        float v = elem<T>::load(x + o);
        for (int j = 0; j < P; ++j) v += a[(size_t)j * d_model + o];
        for (int s = 0; s < n_slices; ++s)
            v += __hip_atomic_load(part + (size_t)s * d_model + o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        elem<T>::store(x_out + o, v);
    }
    if (n_slices > 1 && tid == 0) counters[blockIdx.x] = 0;
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
    int32_t* counters = (int32_t*)(s.ws + s.wl.counters);
    float* q = (float*)(s.ws + s.wl.q);
    float* ctx = (float*)(s.ws + s.wl.ctx);
    float* apart = (float*)(s.ws + s.wl.attn_part);
    float* a = (float*)(s.ws + s.wl.a);
    float* u = (float*)(s.ws + s.wl.u);
    float* dpart = (float*)(s.ws + s.wl.down_part);
    const int bd = s.bypass_d >= P ? P - 1 : s.bypass_d;
    const int xw = (dm + 511) & ~511;

    // counters: [0, P*n_heads) attention units, then the down projection's row blocks
    const int rows_o = 32, rows_d = 32, j_per = 32;
    const int n_att = P * nh;
    const int nrb_d = (dm + rows_d - 1) / rows_d;

    hipLaunchKernelGGL(HIP_KERNEL_NAME(qkv_rope_kernel<T>), dim3(P * 3 * nh), dim3(kThreads),
                       (xw + dk + 16) * sizeof(float), st, (const T*)s.x_in, wqkv, g_attn, rope, s.kv_len, (T*)s.kc,
                       (T*)s.vc, q, counters, s.wl.n_counters, dm, nh, dk, d.max_seq, s.b_max, d.rms_eps);

    int n_chunks = (s.max_kv_len + 1 + kAttnChunk - 1) / kAttnChunk;
    if (n_chunks > s.wl.n_chunks) n_chunks = s.wl.n_chunks;
    if (n_chunks < 1) n_chunks = 1;
    const int lps = dk * (int)sizeof(T) / 16;
    dim3 ga(n_att, n_chunks);
#define CQIL_ATTN(LPS)                                                                                              \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(attn_decode_kernel<T, LPS>), ga, dim3(kThreads), 0, st, q, (const T*)s.kc,   \
                       (const T*)s.vc, s.kv_len, apart, counters, ctx, 1, nh, d.max_seq, s.b_max, s.wl.n_chunks)
    switch (lps) {
        case 4: CQIL_ATTN(4); break;
        case 8: CQIL_ATTN(8); break;
        case 16: CQIL_ATTN(16); break;
        case 32: CQIL_ATTN(32); break;
        default: return hipErrorInvalidValue;
    }
#undef CQIL_ATTN

    hipLaunchKernelGGL(HIP_KERNEL_NAME(oproj_kernel<T>), dim3((dm + rows_o - 1) / rows_o, P), dim3(kThreads),
                       xw * sizeof(float), st, ctx, wo, a, P, dm, rows_o);

    hipLaunchKernelGGL(HIP_KERNEL_NAME(gateup_kernel<T>), dim3((f + j_per - 1) / j_per, P), dim3(kThreads),
                       (xw + 16) * sizeof(float), st, (const T*)s.x_in, a, wgu, g_ffn, u, P, bd, dm, f, j_per,
                       d.rms_eps);

    hipLaunchKernelGGL(HIP_KERNEL_NAME(down_kernel<T>), dim3(nrb_d, s.wl.n_slices), dim3(kThreads),
                       ((s.wl.down_slice + 511) & ~511) * sizeof(float), st, (const T*)s.x_in, a, u, wdown, dpart,
                       counters + n_att, (T*)s.x_out, s.kv_len, s.advance, P, dm, f, rows_d, s.wl.down_slice);
    return hipGetLastError();
}

hipError_t launch_decode_step(const StepArgs& s, hipStream_t st) {
    return s.d.dtype == CQIL_BF16 ? decode_step_t<bf16_t>(s, st) : decode_step_t<float>(s, st);
}

}  // namespace cqil
