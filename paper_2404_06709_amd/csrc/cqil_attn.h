// Kernels shared by the single-token and the small-batch decode paths: attention over the per-layer caches
// and the final merge.
#pragma once
#include "cqil_dev.h"

namespace cqil {

// Attention (Eq.2: softmax(QK^T/sqrt(d_k))V) of one query per workgroup over P independent caches.  One workgroup
// of 16 waves per (layer, token, head): every wave walks the cache in strides, four slot steps (K and V loads of
// all four in flight) per iteration, with a running maximum / sum / context (online softmax); the 16 partial
// results are merged through LDS.  q: element (l, m, h, i) at q[l * q_ls + m * q_ms + h * d_k + i], type QT (fp32
// workspace rows of the decode paths, or the storage-type QKV rows of the token-parallel path); ctx: QT
// [P][M][d_model].  NW waves per workgroup: 16 for few long units, 4 when (layer, token, head) units abound.
// LPS = lanes that share one cache slot = head_dim * sizeof(T) / 16.
constexpr int kAttnThreads = 1024;
constexpr int kAttnWaves = kAttnThreads / kWave;

template <typename T, typename QT, int LPS, int NW>
__global__ __launch_bounds__(NW * 64) void attn_decode_kernel(
    const QT* __restrict__ q, size_t q_ls, size_t q_ms, const T* __restrict__ kc, const T* __restrict__ vc,
    const int32_t* __restrict__ kv_len, QT* __restrict__ ctx, int M, int T_new, int n_heads, int max_seq, int b_max) {
    constexpr int V = elem<T>::kVec;
    constexpr int DK = LPS * V;
    constexpr int SPW = kWave / LPS;  // slots per wave step
    constexpr int U = 4;              // steps per iteration
    __shared__ float red_m[NW], red_l[NW];
    __shared__ float accs[NW][DK];

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int sub = lane % LPS, sg = lane / LPS;
    const int unit = blockIdx.x;
    const int h = unit % n_heads;
    const int lm = unit / n_heads;
    const int m = lm % M, l = lm / M;      // token row m = b * T_new + t
    const int b = m / T_new, t = m % T_new;
    int S = kv_len[b] + t + 1;  // slots to attend: the cache, and the new tokens up to and including this one
    if (S > max_seq) S = max_seq;
    if (S < 1) return;

    const size_t d_model = (size_t)n_heads * DK;
    // scores are kept in units of log 2 (scale = log2 e / sqrt(d_k)): the exponentials are single exp2 instructions
    const float scale = 1.4426950408889634f / sqrtf((float)DK);
    float qv[V];
    {
        const QT* qp = q + (size_t)l * q_ls + (size_t)m * q_ms + (size_t)h * DK + sub * V;
        float qr[V];
        if constexpr (sizeof(QT) * V == 16) {
            elem<QT>::unpack(load16(qp), qr);   // same element type as the cache: one 16-byte load
        } else {
#pragma unroll
            for (int j = 0; j < V; j += 4) {    // fp32 queries: 16-byte loads
                const float4 t = *reinterpret_cast<const float4*>(qp + j);
                qr[j] = t.x; qr[j + 1] = t.y; qr[j + 2] = t.z; qr[j + 3] = t.w;
            }
        }
#pragma unroll
        for (int j = 0; j < V; ++j) qv[j] = qr[j] * scale;
    }
    const size_t head_off = (((size_t)l * b_max + b) * n_heads + h) * (size_t)max_seq * DK;
    const T* kb = kc + head_off + sub * V;
    const T* vb = vc + head_off + sub * V;

    float mx = -INFINITY, lsum = 0.f, acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = 0.f;
    const int n_steps = (S + SPW - 1) / SPW;
    // Software pipeline over the wave's iterations (U slot steps each): the K and V loads of iteration i+1 are
    // requested before iteration i is evaluated, so a wave pays the memory latency once, not once per iteration.
    // Two register sets, the loop advances two iterations per trip (static register indices).
    uint4 kraw[2][U], vraw[2][U];
    auto request = [&](int set, int i0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = (i0 + u) * SPW + sg;
            kraw[set][u] = s < S ? load16_stream(kb + (size_t)s * DK) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = (i0 + u) * SPW + sg;
            vraw[set][u] = s < S ? load16_stream(vb + (size_t)s * DK) : make_uint4(0, 0, 0, 0);
        }
    };
    auto evaluate = [&](int set, int i0) __attribute__((always_inline)) {
        float sc[U], mloc = -INFINITY;
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ok[u] = (i0 + u) * SPW + sg < S;
            float f[V], dot = 0.f;
            elem<T>::unpack(kraw[set][u], f);
#pragma unroll
            for (int j = 0; j < V; ++j) dot = fmaf(f[j], qv[j], dot);
            dot = lane_group_sum<LPS>(dot);
            sc[u] = ok[u] ? dot : -INFINITY;
            mloc = fmaxf(mloc, sc[u]);
        }
        const float nm = fmaxf(mx, mloc);
        if (nm > -INFINITY) {
            const float corr = __builtin_amdgcn_exp2f(mx - nm);  // exp2(-inf) = 0 the first time
            lsum *= corr;
#pragma unroll
            for (int j = 0; j < V; ++j) acc[j] *= corr;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float p = ok[u] ? __builtin_amdgcn_exp2f(sc[u] - nm) : 0.f;
                float f[V];
                elem<T>::unpack(vraw[set][u], f);
                lsum += p;
#pragma unroll
                for (int j = 0; j < V; ++j) acc[j] = fmaf(p, f[j], acc[j]);
            }
            mx = nm;
        }
    };
    constexpr int STRIDE = NW * U;
    int i0 = w * U;
    if (i0 < n_steps) request(0, i0);
    for (; i0 < n_steps; i0 += 2 * STRIDE) {
        if (i0 + STRIDE < n_steps) request(1, i0 + STRIDE);
        evaluate(0, i0);
        if (i0 + STRIDE < n_steps) {
            if (i0 + 2 * STRIDE < n_steps) request(0, i0 + 2 * STRIDE);
            evaluate(1, i0 + STRIDE);
        }
    }
    // merge the slot groups of the wave, then the waves
    float wm = mx;
#pragma unroll
    for (int off = LPS; off < kWave; off <<= 1) wm = fmaxf(wm, __shfl_xor(wm, off, kWave));
    const float sc0 = (mx == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mx - wm);
    lsum *= sc0;
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] *= sc0;
#pragma unroll
    for (int off = LPS; off < kWave; off <<= 1) {
        lsum += __shfl_xor(lsum, off, kWave);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] += __shfl_xor(acc[j], off, kWave);
    }
    if (lane == 0) { red_m[w] = wm; red_l[w] = lsum; }
    if (sg == 0) {
#pragma unroll
        for (int j = 0; j < V; ++j) accs[w][sub * V + j] = acc[j];
    }
    __syncthreads();
    if (tid < DK) {
        float gm = red_m[0];
#pragma unroll
        for (int i = 1; i < NW; ++i) gm = fmaxf(gm, red_m[i]);
        float Ls = 0.f, c = 0.f;
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const float e = (red_m[i] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(red_m[i] - gm);
            Ls += e * red_l[i];
            c += e * accs[i][tid];
        }
        elem<QT>::store(ctx + ((size_t)l * M + m) * d_model + (size_t)h * DK + tid, c / Ls);
    }
}

// Merge of Eq.3 / Eq.4 for one token row: x_out = x + sum_i a_i + sum of the K-slice partials of the down projection;
// also advances the cache lengths.  grid = ceil(d_model / 64) workgroups of 64 x kMergeY threads: thread (tx, ty) adds
// the terms ty, ty + kMergeY, ... of the list [a_0 .. a_{P-1}, part_0 .. part_{n_slices-1}] for output element tx (all
// its loads are requested before the first add), the kMergeY partial sums meet in LDS and are added to x in ty order:
// a fixed order, and one memory latency instead of one per batch of terms.
//   a [P][d_model] fp32, part [n_slices][d_model] fp32
constexpr int kMergeY = 8, kMergeTerms = 8;   // up to kMergeY * kMergeTerms = 64 terms in one pass
template <typename T>
__global__ __launch_bounds__(64 * kMergeY) void merge_kernel(const T* __restrict__ x, const float* __restrict__ a,
                                                             const float* __restrict__ part, T* __restrict__ x_out,
                                                             int32_t* __restrict__ kv_len, int advance, int P,
                                                             int n_slices, int d_model, int B, int T_new) {
    __shared__ float sums[kMergeY][64];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int o = blockIdx.x * 64 + tx;
    const int n_terms = P + n_slices;
    float s = 0.f;
    if (o < d_model) {
        for (int t0 = ty; t0 < n_terms; t0 += kMergeY * kMergeTerms) {
            float t[kMergeTerms];
#pragma unroll
            for (int u = 0; u < kMergeTerms; ++u) {
                const int j = t0 + u * kMergeY;
                t[u] = j < P ? a[(size_t)j * d_model + o] : (j < n_terms ? part[(size_t)(j - P) * d_model + o] : 0.f);
            }
#pragma unroll
            for (int u = 0; u < kMergeTerms; ++u) s += t[u];
        }
    }
    sums[ty][tx] = s;
    __syncthreads();
    if (ty == 0 && o < d_model) {
        float v = elem<T>::load(x + o);
#pragma unroll
        for (int y = 0; y < kMergeY; ++y) v += sums[y][tx];
        elem<T>::store(x_out + o, v);
    }
    if (advance && blockIdx.x == 0)
        for (int b = threadIdx.x; b < B; b += 64 * kMergeY) kv_len[b] += T_new;
}

}  // namespace cqil
