// Token-parallel group step for any batch B and any number of new tokens T (M = B*T token rows), plus the
// model-level kernels (embedding gather, final norm + lm head, greedy argmax).
//
// Steps (same order as the decode path, unfused):
//   rmsnorm_multi   one statistic per token, P gains                          -> nrm [P][M][d_model]
//   gemm (QKV)      grouped over layers                                       -> qkv [M][P*3*d_model]
//   rope_append     rotary embedding of q (in place) and k, KV append
//   attention       causal over cache + new tokens, online softmax            -> ctx [P][M][d_model]
//   gemm (O)        grouped over layers, fp32 output                          -> a   [P][M][d_model]
//   bypass_norm     h_i = x + a_i + window (Eq.4), FFN norms, x + sum a_i      -> nrm, resid
//   gemm (gate/up)  grouped over layers                                       -> gu  [M][P*2*d_ffn]
//   swiglu                                                                    -> u   [M][P*d_ffn]
//   gemm (down)     one contraction over the K-concatenated Wdown + resid     -> x_out
#include "cqil_attn.h"
#include "cqil_dev.h"
#include "cqil_gemv.h"
#include "cqil_internal.h"
#include "cqil_mfma_attn.h"
#include "cqil_mfma_gemm.h"
#include <type_traits>

namespace cqil {

// ------------------------------------------------------------------------------------------ elementwise
// kVec floats -> one 16-byte vector of the storage type
__device__ __forceinline__ uint4 pack16(const float (&f)[4], const float*) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
}
__device__ __forceinline__ uint4 pack16(const float (&f)[8], const bf16_t*) {
    return make_uint4(f32x2_to_bf16x2(f[0], f[1]),
                      f32x2_to_bf16x2(f[2], f[3]),
                      f32x2_to_bf16x2(f[4], f[5]),
                      f32x2_to_bf16x2(f[6], f[7]));
}

// nrm[l][m][k] = x[m][k] * rsqrt(mean x[m]^2 + eps) * g[l][k]; one workgroup per token row, 16-byte accesses
template <typename T>
__global__ __launch_bounds__(1024) void rmsnorm_multi_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                            T* __restrict__ nrm, int P, int M, int d_model, float eps) {
    constexpr int V = elem<T>::kVec;
    __shared__ float scratch[16];
    const int m = blockIdx.x, tid = threadIdx.x;
    const T* xr = x + (size_t)m * d_model;
    const int n_chunks = d_model / V;
    float ss = 0.f;
    for (int c = tid; c < n_chunks; c += blockDim.x) {
        float v[V];
        elem<T>::unpack(load16(xr + c * V), v);
#pragma unroll
        for (int e = 0; e < V; ++e) ss += v[e] * v[e];
    }
    ss = block_sum(ss, scratch);
    const float r = 1.0f / sqrtf(ss / (float)d_model + eps);
    for (int c = tid; c < n_chunks; c += blockDim.x) {
        float v[V];
        elem<T>::unpack(load16(xr + c * V), v);
        for (int l = 0; l < P; ++l) {
            float gv[V], o[V];
            elem<T>::unpack(load16(g + (size_t)l * d_model + c * V), gv);
#pragma unroll
            for (int e = 0; e < V; ++e) o[e] = v[e] * r * gv[e];
            *reinterpret_cast<uint4*>(nrm + ((size_t)l * M + m) * d_model + c * V) = pack16(o, (const T*)nullptr);
        }
    }
}

// Rotary embedding of q (in place) and k, and the KV append, for one token row per workgroup.  A unit is
// (layer, head, chunk of kVec rotary pairs): 16-byte accesses on both halves of the head (d_k / 2 % kVec == 0).
template <typename T>
__global__ __launch_bounds__(1024) void rope_append_kernel(T* __restrict__ qkv, const float2* __restrict__ rope,
                                                          const int32_t* __restrict__ kv_len, T* __restrict__ kc,
                                                          T* __restrict__ vc, int P, int T_new, int n_heads, int d_k,
                                                          int max_seq, int b_max) {
    constexpr int V = elem<T>::kVec;
    const int m = blockIdx.x, b = m / T_new, t = m % T_new;
    const int half = d_k >> 1, cph = half / V;  // chunks per head half
    const int pos = kv_len[b] + t;
    if (pos < 0 || pos >= max_seq) return;
    const size_t d_model = (size_t)n_heads * d_k;
    const int units = P * n_heads * cph;
    for (int u = threadIdx.x; u < units; u += blockDim.x) {
        const int c = u % cph, lh = u / cph, h = lh % n_heads, l = lh / n_heads;
        const int i = c * V;
        T* row = qkv + (size_t)m * P * 3 * d_model + (size_t)l * 3 * d_model + (size_t)h * d_k;
        const size_t slot = ((((size_t)l * b_max + b) * n_heads + h) * max_seq + pos) * d_k;
        float cs[2 * V];
        const float4* rp = reinterpret_cast<const float4*>(rope + (size_t)pos * half + i);
#pragma unroll
        for (int e = 0; e < V / 2; ++e) {
            const float4 r4 = rp[e];
            cs[4 * e] = r4.x; cs[4 * e + 1] = r4.y; cs[4 * e + 2] = r4.z; cs[4 * e + 3] = r4.w;
        }
        float lo[V], hi[V], olo[V], ohi[V];
        elem<T>::unpack(load16(row + i), lo);
        elem<T>::unpack(load16(row + i + half), hi);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            olo[e] = lo[e] * cs[2 * e] - hi[e] * cs[2 * e + 1];
            ohi[e] = hi[e] * cs[2 * e] + lo[e] * cs[2 * e + 1];
        }
        *reinterpret_cast<uint4*>(row + i) = pack16(olo, (const T*)nullptr);
        *reinterpret_cast<uint4*>(row + i + half) = pack16(ohi, (const T*)nullptr);
        const T* kr = row + d_model;
        elem<T>::unpack(load16(kr + i), lo);
        elem<T>::unpack(load16(kr + i + half), hi);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            olo[e] = lo[e] * cs[2 * e] - hi[e] * cs[2 * e + 1];
            ohi[e] = hi[e] * cs[2 * e] + lo[e] * cs[2 * e + 1];
        }
        *reinterpret_cast<uint4*>(kc + slot + i) = pack16(olo, (const T*)nullptr);
        *reinterpret_cast<uint4*>(kc + slot + i + half) = pack16(ohi, (const T*)nullptr);
        const T* vr = row + 2 * d_model;
        *reinterpret_cast<uint4*>(vc + slot + i) = load16(vr + i);
        *reinterpret_cast<uint4*>(vc + slot + i + half) = load16(vr + i + half);
    }
}

// Attention of one query (token m, layer l, head h) over slots 0 .. kv_len[b]+t, online softmax.
// grid = (M, P*n_heads), 256 threads; LPS lanes share one cache slot.
template <typename T, int LPS>
__global__ __launch_bounds__(256) void attn_generic_kernel(const T* __restrict__ qkv, const T* __restrict__ kc,
                                                            const T* __restrict__ vc,
                                                            const int32_t* __restrict__ kv_len, T* __restrict__ ctx,
                                                            int P, int M, int T_new, int n_heads, int max_seq,
                                                            int b_max) {
    constexpr int V = elem<T>::kVec;
    constexpr int DK = LPS * V;
    constexpr int SPW = kWave / LPS;
    __shared__ float red_m[4], red_l[4];
    __shared__ float accs[4][DK];
    const int m = blockIdx.x, b = m / T_new, t = m % T_new;
    const int lh = blockIdx.y, l = lh / n_heads, h = lh % n_heads;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int sub = lane % LPS, sg = lane / LPS;
    int S = kv_len[b] + t + 1;
    if (S > max_seq) S = max_seq;
    const size_t d_model = (size_t)n_heads * DK;
    T* out = ctx + ((size_t)l * M + m) * d_model + (size_t)h * DK;
    if (S < 1) return;
    const float scale = 1.0f / sqrtf((float)DK);
    float qv[V];
    {
        float f[V];
        elem<T>::unpack(load16(qkv + (size_t)m * P * 3 * d_model + (size_t)l * 3 * d_model + (size_t)h * DK + sub * V), f);
#pragma unroll
        for (int j = 0; j < V; ++j) qv[j] = f[j] * scale;
    }
    const size_t head_off = (((size_t)l * b_max + b) * n_heads + h) * (size_t)max_seq * DK;
    const T* kb = kc + head_off;
    const T* vb = vc + head_off;
    float mx = -INFINITY, lsum = 0.f, acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = 0.f;
    for (int s = w * SPW + sg; s < S; s += 4 * SPW) {
        // the LPS lanes of a slot group run this loop together (s depends on lane only through sg)
        float f[V], dot = 0.f;
        elem<T>::unpack(load16(kb + (size_t)s * DK + sub * V), f);
#pragma unroll
        for (int j = 0; j < V; ++j) dot = fmaf(f[j], qv[j], dot);
#pragma unroll
        for (int off = LPS / 2; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, kWave);
        const float nm = fmaxf(mx, dot);
        const float corr = expf(mx - nm), p = expf(dot - nm);   // exp(-inf) = 0 on the first slot
        elem<T>::unpack(load16(vb + (size_t)s * DK + sub * V), f);
        lsum = lsum * corr + p;
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] = fmaf(p, f[j], acc[j] * corr);
        mx = nm;
    }
    // merge the slot groups of the wave, then the waves
    float wm = mx;
#pragma unroll
    for (int off = LPS; off < kWave; off <<= 1) wm = fmaxf(wm, __shfl_xor(wm, off, kWave));
    const float sc = (mx == -INFINITY) ? 0.f : expf(mx - wm);
    lsum *= sc;
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] *= sc;
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
        for (int i = 1; i < 4; ++i) gm = fmaxf(gm, red_m[i]);
        float L = 0.f, c = 0.f;
        for (int i = 0; i < 4; ++i) {
            const float e = (red_m[i] == -INFINITY) ? 0.f : expf(red_m[i] - gm);
            L += e * red_l[i];
            c += e * accs[i][tid];
        }
        elem<T>::store(out + tid, c / L);
    }
}

// Bypass window, FFN norms and the residual carrier for one token row per workgroup:
//   h_i = x + sum_{j=max(0,i-d)}^{i} a_j ; nrm_i = RMSNorm(h_i) g_i ; resid = xres + sum_j a_j
// (xres is x itself except under input substitution, where the branches computed from x are added to another state)
// 16-byte accesses: a thread owns chunks of kVec consecutive elements (d_model % kVec == 0).
template <typename T>
__global__ __launch_bounds__(1024) void bypass_norm_kernel(const T* __restrict__ x, const T* __restrict__ xres,
                                                          const float* __restrict__ a,
                                                          const T* __restrict__ g_ffn, T* __restrict__ nrm,
                                                          float* __restrict__ resid, int P, int bypass_d, int M,
                                                          int d_model, float eps, int32_t* __restrict__ kv_len,
                                                          int advance_B, int advance_T) {
    constexpr int V = elem<T>::kVec;
    __shared__ float scratch[16];
    const int m = blockIdx.x, tid = threadIdx.x;
    const T* xr = x + (size_t)m * d_model;
    const T* xrr = xres + (size_t)m * d_model;
    const int n_chunks = d_model / V;
    // h_i for the chunk at k: x plus the window of attention outputs
    auto window = [&](const T* base, int k, int jlo, int jhi, float (&hv)[V]) {
        elem<T>::unpack(load16(base + k), hv);
        for (int j = jlo; j <= jhi; ++j) {
            const float* ap = a + ((size_t)j * M + m) * d_model + k;
#pragma unroll
            for (int e = 0; e < V; e += 4) {
                const float4 t = *reinterpret_cast<const float4*>(ap + e);
                hv[e] += t.x; hv[e + 1] += t.y; hv[e + 2] += t.z; hv[e + 3] += t.w;
            }
        }
    };
    for (int i = 0; i < P; ++i) {
        const int jlo = bypass_d < 0 ? i + 1 : max(0, i - bypass_d);  // negative: Eq.5, the input is x alone
        float ss = 0.f;
        for (int c = tid; c < n_chunks; c += blockDim.x) {
            float hv[V];
            window(xr, c * V, jlo, i, hv);
#pragma unroll
            for (int e = 0; e < V; ++e) ss += hv[e] * hv[e];
        }
        ss = block_sum(ss, scratch);
        const float r = 1.0f / sqrtf(ss / (float)d_model + eps);
        const T* gi = g_ffn + (size_t)i * d_model;
        T* out = nrm + ((size_t)i * M + m) * d_model;
        for (int c = tid; c < n_chunks; c += blockDim.x) {
            float hv[V], gv[V];
            window(xr, c * V, jlo, i, hv);
            elem<T>::unpack(load16(gi + c * V), gv);
#pragma unroll
            for (int e = 0; e < V; ++e) hv[e] = hv[e] * r * gv[e];
            *reinterpret_cast<uint4*>(out + c * V) = pack16(hv, (const T*)nullptr);
        }
    }
    // every reader of the cache lengths (rotary/append, attention) ran before this kernel: advance them here
    if (advance_B > 0 && m == 0)
        for (int b = tid; b < advance_B; b += blockDim.x) kv_len[b] += advance_T;
    for (int c = tid; c < n_chunks; c += blockDim.x) {
        float hv[V];
        window(xrr, c * V, 0, P - 1, hv);
#pragma unroll
        for (int e = 0; e < V; e += 4)
            *reinterpret_cast<float4*>(resid + (size_t)m * d_model + c * V + e) = make_float4(hv[e], hv[e + 1], hv[e + 2], hv[e + 3]);
    }
}

// The same for rows of at most 1024 16-byte chunks and groups of at most 8 layers: a thread owns one chunk, reads x
// and the P attention outputs of it once and keeps them in registers, so the row crosses the memory system once
// (the general kernel re-reads the window in every pass).  blockDim.x >= d_model / V, a multiple of 64.
constexpr int kBypassRegLayers = 8;
template <typename T>
__global__ __launch_bounds__(1024) void bypass_norm_reg_kernel(const T* __restrict__ x, const T* __restrict__ xres,
                                                              const float* __restrict__ a,
                                                              const T* __restrict__ g_ffn, T* __restrict__ nrm,
                                                              float* __restrict__ resid, int P, int bypass_d, int M,
                                                              int d_model, float eps, int32_t* __restrict__ kv_len,
                                                              int advance_B, int advance_T) {
    constexpr int V = elem<T>::kVec;
    __shared__ float scratch[16 * kBypassRegLayers];   // [wave][layer]
    const int m = blockIdx.x, tid = threadIdx.x;
    const bool act = tid < d_model / V;
    const int k = act ? tid * V : 0;
    float xv[V], av[kBypassRegLayers][V];
    elem<T>::unpack(load16(x + (size_t)m * d_model + k), xv);
#pragma unroll
    for (int j = 0; j < kBypassRegLayers; ++j) {
        if (j < P) {
            const float* ap = a + ((size_t)j * M + m) * d_model + k;
#pragma unroll
            for (int e = 0; e < V; e += 4) {
                const float4 t = *reinterpret_cast<const float4*>(ap + e);
                av[j][e] = t.x; av[j][e + 1] = t.y; av[j][e + 2] = t.z; av[j][e + 3] = t.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) av[j][e] = 0.f;
        }
    }
    // the P sums of squares are reduced together: one pass through LDS (two barriers) for the whole group
    float ssq[kBypassRegLayers];
#pragma unroll
    for (int i = 0; i < kBypassRegLayers; ++i) {
        ssq[i] = 0.f;
        if (i >= P) continue;
        const int jlo = bypass_d < 0 ? i + 1 : max(0, i - bypass_d);  // negative: Eq.5, the input is x alone
        float hv[V];
#pragma unroll
        for (int e = 0; e < V; ++e) hv[e] = xv[e];
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            if (j >= jlo) {
#pragma unroll
                for (int e = 0; e < V; ++e) hv[e] += av[j][e];
            }
        }
        if (act) {
#pragma unroll
            for (int e = 0; e < V; ++e) ssq[i] += hv[e] * hv[e];
        }
        ssq[i] = wave_sum(ssq[i]);
    }
    const int wv = tid >> 6, nw = blockDim.x >> 6;
    if ((tid & 63) == 0) {
#pragma unroll
        for (int i = 0; i < kBypassRegLayers; ++i) scratch[wv * kBypassRegLayers + i] = ssq[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kBypassRegLayers; ++i) {
        if (i >= P) break;
        float tot = 0.f;
        for (int ww = 0; ww < nw; ++ww) tot += scratch[ww * kBypassRegLayers + i];
        const float r = 1.0f / sqrtf(tot / (float)d_model + eps);
        if (act) {
            const int jlo = bypass_d < 0 ? i + 1 : max(0, i - bypass_d);
            float hv[V], gv[V];
#pragma unroll
            for (int e = 0; e < V; ++e) hv[e] = xv[e];
#pragma unroll
            for (int j = 0; j <= i; ++j) {
                if (j >= jlo) {
#pragma unroll
                    for (int e = 0; e < V; ++e) hv[e] += av[j][e];
                }
            }
            elem<T>::unpack(load16(g_ffn + (size_t)i * d_model + k), gv);
#pragma unroll
            for (int e = 0; e < V; ++e) hv[e] = hv[e] * r * gv[e];
            *reinterpret_cast<uint4*>(nrm + ((size_t)i * M + m) * d_model + k) = pack16(hv, (const T*)nullptr);
        }
    }
    if (advance_B > 0 && m == 0)
        for (int b = tid; b < advance_B; b += blockDim.x) kv_len[b] += advance_T;
    if (act) {
        if (xres != x) elem<T>::unpack(load16(xres + (size_t)m * d_model + k), xv);  // wave-uniform
#pragma unroll
        for (int j = 0; j < kBypassRegLayers; ++j)
#pragma unroll
            for (int e = 0; e < V; ++e) xv[e] += av[j][e];  // layers past P hold zeros
#pragma unroll
        for (int e = 0; e < V; e += 4)
            *reinterpret_cast<float4*>(resid + (size_t)m * d_model + k + e) = make_float4(xv[e], xv[e + 1], xv[e + 2], xv[e + 3]);
    }
}

// u[m][l*f + j] = silu(gate) * up, reading the block-interleaved gate/up columns
template <typename T>
__global__ void swiglu_kernel(const T* __restrict__ gu, T* __restrict__ u, int P, int M, int d_ffn) {
    const size_t total = (size_t)M * P * d_ffn;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t m = i / ((size_t)P * d_ffn);
        const int lj = (int)(i % ((size_t)P * d_ffn));
        const int l = lj / d_ffn, j = lj % d_ffn;
        const T* row = gu + m * (size_t)P * 2 * d_ffn + (size_t)l * 2 * d_ffn + (size_t)(j / kGuBlock) * 2 * kGuBlock + j % kGuBlock;
        const float g = elem<T>::load(row), up = elem<T>::load(row + kGuBlock);
        elem<T>::store(u + i, g / (1.0f + expf(-g)) * up);
    }
}

// ------------------------------------------------------------------------------------------ plain GEMM
// C[m][n] = sum_k A[m][k] * B[n][k]  (+ R[m][n]), fp32 accumulate, 64x64 tile, 16-wide K steps, 4x4 per thread.
// A and C are row-major; B is a packed weight matrix in the tiled layout with padded width Kp.  blockIdx.z selects
// a group: A and C advance by element strides, B by a row offset and a column offset (N- or K-concatenation).
// K % 4 == 0.
template <typename AT, typename BT, typename CT, bool ADD_R>
__global__ __launch_bounds__(256) void gemm_nt_kernel(const AT* __restrict__ A, const BT* __restrict__ B,
                                                      CT* __restrict__ C, const float* __restrict__ R, int M, int N,
                                                      int K, size_t lda, size_t Kp, size_t ldc, size_t sA,
                                                      size_t n_step, size_t k_step, size_t sC) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    A += (size_t)blockIdx.z * sA; C += (size_t)blockIdx.z * sC;
    const size_t n_off = (size_t)blockIdx.z * n_step, k_off = (size_t)blockIdx.z * k_step;
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tx = tid % 16, ty = tid / 16;
    const int lr = tid / 4, lc = (tid % 4) * 4;  // loader: row lr of the tile, 4 consecutive k
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        {
            const int gm = m0 + lr, gk = k0 + lc;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (gm < M && gk < K)
                for (int j = 0; j < 4; ++j) v[j] = elem<AT>::load(A + (size_t)gm * lda + gk + j);
            for (int j = 0; j < 4; ++j) As[lc + j][lr] = v[j];
        }
        {
            const int gn = n0 + lr, gk = k0 + lc;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (gn < N && gk < K)
            {
                // four consecutive columns of one row lie inside one 16-byte piece of a tile
                const BT* bp = B + tile<BT>::offset(n_off + gn, k_off + gk, Kp);
                for (int j = 0; j < 4; ++j) v[j] = elem<BT>::load(bp + j);
            }
            for (int j = 0; j < 4; ++j) Bs[lc + j][lr] = v[j];
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc[i][j];
            if (ADD_R) v += R[(size_t)gm * N + gn];
            elem<CT>::store(C + (size_t)gm * ldc + gn, v);
        }
    }
}

template <typename AT, typename BT, typename CT, bool ADD_R>
static void gemm_nt(const AT* A, const BT* B, CT* C, const float* R, int M, int N, int K, size_t lda, size_t Kp,
                    size_t ldc, int groups, size_t sA, size_t n_step, size_t k_step, size_t sC, hipStream_t st) {
    dim3 grid((N + 63) / 64, (M + 63) / 64, groups);
    hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_nt_kernel<AT, BT, CT, ADD_R>), grid, dim3(256), 0, st, A, B, C, R, M, N, K,
                       lda, Kp, ldc, sA, n_step, k_step, sC);
}

// bf16 products run on the matrix cores, fp32 ones on the plain kernel above.  part / part_floats: scratch for
// split-K partial sums of the matrix-core kernel (null: never split).
template <typename T, typename CT, bool ADD_R>
static hipError_t gemm_any(const T* A, const T* W, CT* C, const float* R, int M, int N, int K, size_t lda, size_t Kp,
                           size_t ldc, int groups, size_t sA, size_t n_step, size_t k_step, size_t sC, hipStream_t st,
                           float* part = nullptr, size_t part_floats = 0) {
    if constexpr (std::is_same<T, bf16_t>::value) {
        return gemm_mfma<CT, ADD_R ? kEpiAddR : kEpiNone>(g_tune.gemm_tile.load(), A, W, C, R, M, N, K, lda, Kp, ldc, groups, sA,
                                                          n_step, k_step, sC, st, part, part_floats);
    } else {
        gemm_nt<T, T, CT, ADD_R>(A, W, C, R, M, N, K, lda, Kp, ldc, groups, sA, n_step, k_step, sC, st);
        return hipSuccess;
    }
}

__global__ void advance_kernel(int32_t* kv_len, int B, int T) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) kv_len[b] += T;
}

__global__ void copy16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

hipError_t launch_copy16(const void* src, void* dst, size_t bytes, hipStream_t st) {
    const size_t n = bytes / 16;
    const unsigned grid = (unsigned)((n + 255) / 256 > 4096 ? 4096 : (n + 255) / 256);
    hipLaunchKernelGGL(copy16_kernel, dim3(grid ? grid : 1), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n);
    return hipGetLastError();
}

hipError_t launch_advance(int32_t* kv_len, int B, int T, hipStream_t st) {
    hipLaunchKernelGGL(advance_kernel, dim3((B + 63) / 64), dim3(64), 0, st, kv_len, B, T);
    return hipGetLastError();
}

template <typename T>
static hipError_t generic_step_t(const StepArgs& s, hipStream_t st) {
    const cqil_dims& d = s.d;
    const int P = s.P, dm = d.d_model, f = d.d_ffn, dk = d.head_dim, nh = d.n_heads;
    const int M = s.B * s.T;
    const T* wqkv = (const T*)(s.packed + s.pl.wqkv);
    const T* wo = (const T*)(s.packed + s.pl.wo);
    const T* wgu = (const T*)(s.packed + s.pl.wgu);
    const T* wdown = (const T*)(s.packed + s.pl.wdown);
    const T* g_attn = (const T*)(s.packed + s.pl.g_attn);
    const T* g_ffn = (const T*)(s.packed + s.pl.g_ffn);
    const float2* rope = (const float2*)(s.packed + s.pl.rope);
    T* nrm = (T*)(s.ws + s.wl.nrm);
    T* qkv = (T*)(s.ws + s.wl.qkv);
    T* ctx = (T*)(s.ws + s.wl.ctx_act);
    float* a = (float*)(s.ws + s.wl.a);
    float* resid = (float*)(s.ws + s.wl.resid);
    T* gu = (T*)(s.ws + s.wl.gu);
    T* u = (T*)(s.ws + s.wl.u_act);
    const T* x = (const T*)s.x_in;
    const int bd = s.bypass_d >= P ? P - 1 : s.bypass_d;
    const size_t Mdm = (size_t)M * dm;

    const int row_threads = M <= 64 ? 1024 : 256;  // few rows: more threads per row, the kernels are latency-bound
    hipLaunchKernelGGL(HIP_KERNEL_NAME(rmsnorm_multi_kernel<T>), dim3(M), dim3(row_threads), 0, st, x, g_attn, nrm, P, M,
                       dm, d.rms_eps);
    hipError_t ge;
    float* part = s.wl.gemm_part_floats ? (float*)(s.ws + s.wl.gemm_part) : nullptr;
    // Prefill-sized bf16 products of the LLaMA head sizes: the rotary embedding and the KV append run in the epilogue
    // of the QKV product (q goes to the QKV rows, k and v straight into the caches); otherwise a separate pass.
    bool rope_fused = false;
    if constexpr (std::is_same<T, bf16_t>::value) {
        if (M >= 512 && dm % 256 == 0 && (dk == 64 || dk == 128) && g_tune.gemm_tile.load() == 0) {
            GemmRope rp;
            rp.rope = rope; rp.kv_len = s.kv_len; rp.kc = (bf16_t*)s.kc; rp.vc = (bf16_t*)s.vc;
            rp.T_new = s.T; rp.n_heads = nh; rp.d_k = dk; rp.max_seq = d.max_seq; rp.b_max = s.b_max; rp.d_model = dm;
            if ((ge = gemm_mfma_qkv_rope(nrm, wqkv, qkv, M, 3 * dm, dm, dm, dm, (size_t)P * 3 * dm, P, Mdm, (size_t)3 * dm,
                                         (size_t)3 * dm, rp, st)) != hipSuccess) return ge;
            rope_fused = true;
        }
    }
    if (!rope_fused) {
        if ((ge = gemm_any<T, T, false>(nrm, wqkv, qkv, nullptr, M, 3 * dm, dm, dm, dm, (size_t)P * 3 * dm, P, Mdm,
                                (size_t)3 * dm, 0, (size_t)3 * dm, st, part, s.wl.gemm_part_floats)) != hipSuccess) return ge;
        hipLaunchKernelGGL(HIP_KERNEL_NAME(rope_append_kernel<T>), dim3(M), dim3(row_threads), 0, st,
                           qkv, rope, s.kv_len, (T*)s.kc, (T*)s.vc, P, s.T, nh, dk, d.max_seq, s.b_max);
    }
    const int lps = dk * (int)sizeof(T) / 16;
    bool attn_done = false;
    if (s.T == 1) {
        // one query per sequence: the streaming kernel of the decode paths, reading q from the QKV rows; four
        // waves per (layer, sequence, head) once those units outnumber the CUs several times over
        const bool many = (long)P * M * nh >= 2048;
#define CQIL_ATTN1(LPS)                                                                                                \
    if (many)                                                                                                          \
        hipLaunchKernelGGL(HIP_KERNEL_NAME(attn_decode_kernel<T, T, LPS, 4>), dim3(P * M * nh), dim3(256), 0, st,         \
                           (const T*)qkv, (size_t)3 * dm, (size_t)P * 3 * dm, (const T*)s.kc, (const T*)s.vc, s.kv_len, ctx, \
                           M, 1, nh, d.max_seq, s.b_max);                                                              \
    else                                                                                                               \
        hipLaunchKernelGGL(HIP_KERNEL_NAME(attn_decode_kernel<T, T, LPS, kAttnWaves>), dim3(P * M * nh),                   \
                           dim3(kAttnThreads), 0, st, (const T*)qkv, (size_t)3 * dm, (size_t)P * 3 * dm, (const T*)s.kc,    \
                           (const T*)s.vc, s.kv_len, ctx, M, 1, nh, d.max_seq, s.b_max)
        switch (lps) {
            case 4: CQIL_ATTN1(4); break;
            case 8: CQIL_ATTN1(8); break;
            case 16: CQIL_ATTN1(16); break;
            case 32: CQIL_ATTN1(32); break;
            case 64: CQIL_ATTN1(64); break;
            default: return hipErrorInvalidValue;
        }
#undef CQIL_ATTN1
        attn_done = true;
    }
    if constexpr (std::is_same<T, bf16_t>::value) {
        // matrix-core attention for the head sizes it is built for; positions were bounded by the caller
        if (!attn_done && (dk == 64 || dk == 128)) {
            // 1-D grid: 8 XCDs x groups of kPfUnitGroup head units x query blocks (the kernel skips the padding)
            const int nqb = (s.T + kPfBQ - 1) / kPfBQ, units_per_xcd = (P * s.B * nh + 7) / 8;
            const dim3 grid(8u * ((units_per_xcd + kPfUnitGroup - 1) / kPfUnitGroup) * kPfUnitGroup * nqb);
            const bool old_form = g_tune.attn_prefill.load() == 1;  // 16x16x32 instructions (the slower form)
#define CQIL_PF(KERNEL)                                                                                                  \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(KERNEL), grid, dim3(kPfThreads), 0, st, (const bf16_t*)qkv, (const bf16_t*)s.kc,    \
                       (const bf16_t*)s.vc, s.kv_len, ctx, P, s.B, s.T, nh, d.max_seq, s.b_max)
            if (dk == 64) {
                if (old_form) CQIL_PF(attn_prefill_mfma_kernel<64>); else CQIL_PF(attn_prefill_mfma32_kernel<64>);
            } else {
                if (old_form) CQIL_PF(attn_prefill_mfma_kernel<128>); else CQIL_PF(attn_prefill_mfma32_kernel<128>);
            }
#undef CQIL_PF
            attn_done = true;
        }
    }
    if (!attn_done) {
#define CQIL_ATTN(LPS)                                                                                               \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(attn_generic_kernel<T, LPS>), dim3(M, P * nh), dim3(256), 0, st, (const T*)qkv, \
                       (const T*)s.kc, (const T*)s.vc, s.kv_len, ctx, P, M, s.T, nh, d.max_seq, s.b_max)
    switch (lps) {
        case 4: CQIL_ATTN(4); break;
        case 8: CQIL_ATTN(8); break;
        case 16: CQIL_ATTN(16); break;
        case 32: CQIL_ATTN(32); break;
        case 64: CQIL_ATTN(64); break;
        default: return hipErrorInvalidValue;
    }
#undef CQIL_ATTN
    }
    if ((ge = gemm_any<T, float, false>(ctx, wo, a, nullptr, M, dm, dm, dm, (size_t)P * dm, dm, P, Mdm, 0, (size_t)dm, Mdm, st,
                                        part, s.wl.gemm_part_floats)) != hipSuccess) return ge;
    if (P <= kBypassRegLayers && dm / elem<T>::kVec <= 1024)
        hipLaunchKernelGGL(HIP_KERNEL_NAME(bypass_norm_reg_kernel<T>), dim3(M), dim3((dm / elem<T>::kVec + 63) / 64 * 64), 0,
                           st, x, (const T*)s.x_res, a, g_ffn, nrm, resid, P, bd, M, dm, d.rms_eps, s.kv_len, s.advance ? s.B : 0, s.T);
    else
        hipLaunchKernelGGL(HIP_KERNEL_NAME(bypass_norm_kernel<T>), dim3(M), dim3(row_threads), 0, st, x, (const T*)s.x_res, a, g_ffn, nrm,
                           resid, P, bd, M, dm, d.rms_eps, s.kv_len, s.advance ? s.B : 0, s.T);
    if constexpr (std::is_same<T, bf16_t>::value) {
        // gate/up product with SwiGLU in the epilogue: u is written directly, gate and up never reach memory
        if ((ge = gemm_mfma<bf16_t, kEpiSwiglu>(g_tune.gemm_tile.load(), nrm, wgu, u, nullptr, M, 2 * f, dm, dm, dm, (size_t)P * f,
                                                 P, Mdm, (size_t)2 * f, 0, (size_t)f, st)) != hipSuccess) return ge;
    } else {
        if ((ge = gemm_any<T, T, false>(nrm, wgu, gu, nullptr, M, 2 * f, dm, dm, dm, (size_t)P * 2 * f, P, Mdm, (size_t)2 * f, 0,
                                (size_t)2 * f, st)) != hipSuccess) return ge;
        const size_t total = (size_t)M * P * f;
        size_t g = (total + 255) / 256;
        if (g > 65536) g = 65536;
        hipLaunchKernelGGL(HIP_KERNEL_NAME(swiglu_kernel<T>), dim3((int)g), dim3(256), 0, st, (const T*)gu, u, P, M, f);
    }
    {
        const size_t kt = tile<T>::KB, Kp = ((size_t)P * f + kt - 1) / kt * kt;
        if ((ge = gemm_any<T, T, true>(u, wdown, (T*)s.x_out, resid, M, dm, P * f, (size_t)P * f, Kp, dm, 1, 0, 0, 0, 0, st, part,
                                       s.wl.gemm_part_floats)) != hipSuccess) return ge;
    }
    return hipGetLastError();
}

hipError_t launch_generic_step(const StepArgs& s, hipStream_t st) {
    return s.d.dtype == CQIL_BF16 ? generic_step_t<bf16_t>(s, st) : generic_step_t<float>(s, st);
}

// ------------------------------------------------------------------------------------------ model level
template <typename T>
__global__ void embedding_kernel(const T* __restrict__ emb, const int32_t* __restrict__ tokens, T* __restrict__ x,
                                 int M, int vocab, int vec_per_row) {
    const int m = blockIdx.x;
    int tok = tokens[m];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);  // never read outside the table
    const uint4* src = reinterpret_cast<const uint4*>(emb) + (size_t)tok * vec_per_row;
    uint4* dst = reinterpret_cast<uint4*>(x) + (size_t)m * vec_per_row;
    for (int i = threadIdx.x; i < vec_per_row; i += blockDim.x) dst[i] = src[i];
}

hipError_t launch_embedding(const cqil_dims& d, const void* emb, const int32_t* tokens, int M, int vocab, void* x,
                            hipStream_t st) {
    const int vpr = d.d_model * (int)esize(d.dtype) / 16;
    if (d.dtype == CQIL_BF16)
        hipLaunchKernelGGL(HIP_KERNEL_NAME(embedding_kernel<bf16_t>), dim3(M), dim3(256), 0, st, (const bf16_t*)emb,
                           tokens, (bf16_t*)x, M, vocab, vpr);
    else
        hipLaunchKernelGGL(HIP_KERNEL_NAME(embedding_kernel<float>), dim3(M), dim3(256), 0, st, (const float*)emb,
                           tokens, (float*)x, M, vocab, vpr);
    return hipGetLastError();
}

// logits[b][v] = lm_head[v] . RMSNorm(hidden[b][T-1]) g_final.  grid = (row blocks of the vocabulary, B)
template <typename T>
__global__ __launch_bounds__(kThreads) void head_kernel(const T* __restrict__ hidden, const T* __restrict__ g_final,
                                                         const T* __restrict__ lm_head, float* __restrict__ logits,
                                                         int T_new, int d_model, int vocab, int rows_per_wg, float eps) {
    extern __shared__ float smem[];
    constexpr int V = elem<T>::kVec;
    float* xs = smem;
    float* scratch = xs + xs_words(d_model);
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int b = blockIdx.y;
    const T* x = hidden + ((size_t)b * T_new + (T_new - 1)) * d_model;
    float ss = 0.f;
    for (int k = tid; k < d_model; k += kThreads) {
        const float v = elem<T>::load(x + k);
        ss += v * v;
    }
    ss = block_sum(ss, scratch);
    const float r = 1.0f / sqrtf(ss / (float)d_model + eps);
    for (int k = tid; k < d_model; k += kThreads) xs[xs_index<V>(k)] = elem<T>::load(x + k) * r * elem<T>::load(g_final + k);
    __syncthreads();
    const int row0 = blockIdx.x * rows_per_wg;
    const int row1 = min(row0 + rows_per_wg, vocab);
    for (int o = row0 + 4 * w; o < row1; o += 4 * kWaves) {
        // the last group of a vocabulary that is not a multiple of 4 re-reads the last row
        const int o1 = min(o + 1, vocab - 1), o2 = min(o + 2, vocab - 1), o3 = min(o + 3, vocab - 1);
        float s[4];
        dot4<T>(lm_head + (size_t)o * d_model, lm_head + (size_t)o1 * d_model, lm_head + (size_t)o2 * d_model,
                lm_head + (size_t)o3 * d_model, xs, d_model, s);
        if (lane == 0) {
            float* out = logits + (size_t)b * vocab;
            out[o] = s[0];
            if (o + 1 < vocab) out[o + 1] = s[1];
            if (o + 2 < vocab) out[o + 2] = s[2];
            if (o + 3 < vocab) out[o + 3] = s[3];
        }
    }
}

// greedy token: lowest index among the maxima.  One workgroup of 1024 threads per sequence; 16-byte loads when the
// rows allow it.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits, int32_t* __restrict__ next, int vocab) {
    __shared__ float bv[1024];
    __shared__ int bi[1024];
    const int b = blockIdx.x, tid = threadIdx.x;
    const float* lg = logits + (size_t)b * vocab;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    auto take = [&](float x, int v) {
        if (x > best || (x == best && v < idx)) { best = x; idx = v; }
    };
    if ((vocab & 3) == 0 && (((uintptr_t)logits) & 15) == 0) {
        for (int v = 4 * tid; v < vocab; v += 4096) {
            const float4 x = *reinterpret_cast<const float4*>(lg + v);
            take(x.x, v); take(x.y, v + 1); take(x.z, v + 2); take(x.w, v + 3);
        }
    } else {
        for (int v = tid; v < vocab; v += 1024) take(lg[v], v);
    }
    bv[tid] = best; bi[tid] = idx;
    __syncthreads();
    for (int s = 512; s >= 1; s >>= 1) {
        if (tid < s) {
            const float ov = bv[tid + s];
            const int oi = bi[tid + s];
            if (ov > bv[tid] || (ov == bv[tid] && oi < bi[tid])) { bv[tid] = ov; bi[tid] = oi; }
        }
        __syncthreads();
    }
    if (tid == 0) next[b] = bi[0] == 0x7fffffff ? 0 : bi[0];
}

hipError_t launch_head(const HeadArgs& h, hipStream_t st) {
    const int rows = 32;
    const int xw = (h.d.d_model + 511) & ~511;
    dim3 grid((h.vocab + rows - 1) / rows, h.B);
    if (h.d.dtype == CQIL_BF16)
        hipLaunchKernelGGL(HIP_KERNEL_NAME(head_kernel<bf16_t>), grid, dim3(kThreads), (xw + 16) * sizeof(float), st,
                           (const bf16_t*)h.hidden, (const bf16_t*)h.g_final, (const bf16_t*)h.lm_head, h.logits, h.T,
                           h.d.d_model, h.vocab, rows, h.d.rms_eps);
    else
        hipLaunchKernelGGL(HIP_KERNEL_NAME(head_kernel<float>), grid, dim3(kThreads), (xw + 16) * sizeof(float), st,
                           (const float*)h.hidden, (const float*)h.g_final, (const float*)h.lm_head, h.logits, h.T,
                           h.d.d_model, h.vocab, rows, h.d.rms_eps);
    if (h.next_token) hipLaunchKernelGGL(argmax_kernel, dim3(h.B), dim3(1024), 0, st, h.logits, h.next_token, h.vocab);
    return hipGetLastError();
}

}  // namespace cqil
