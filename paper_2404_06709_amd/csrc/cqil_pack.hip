// cqil_pack_group: one-time packing of P layers' weights into the group layout.
//
// The paper places layer l+i of a group on GPU i (Alg.1).  On one GPU the same independence is expressed by
// concatenation: projections that read the shared input (Wq, Wk, Wv; Wgate, Wup) are stacked along their output
// dimension, and the projections whose results Eq.3 / Eq.4 sum over the group (Wo, Wdown) are laid side by side
// along their input dimension, so that the sum over layers is part of one long dot product.  Each concatenated
// matrix is then stored in 1 KiB tiles of 16 rows (see tile<> in cqil_dev.h) so that a 64-lane wave streams it with
// fully contiguous 16-byte loads and receives matrix-core operand fragments directly.  Everything here is a pure
// index map on 16-byte pieces (8 bf16 or 4 fp32 values of one source row); padding columns are zero.
#include "cqil_dev.h"
#include "cqil_internal.h"

namespace cqil {

struct PackPtrs {
    const char* p[kMaxP];
};

enum PackKind { kPackQkv = 0, kPackWo = 1, kPackGu = 2, kPackDown = 3 };

// One thread per destination 16-byte piece.  The destination piece index decomposes as
// (row strip rt, k block kb, k group g, row in strip i); logical row r = 16 rt + i, first column k = KB kb + V g.
//   kPackQkv : rows [l][q|k|v][o], K = d_model          source row o of W_m of layer l
//   kPackWo  : rows o, K = [l][d_model]                 source row o of Wo of layer l
//   kPackGu  : rows [l][j/16][gate|up][j%16], K = d_model
//   kPackDown: rows o, K = [l][d_ffn] (+ zero padding)  source row o of Wdown of layer l
template <int KIND, int V>
__global__ void pack_tiled_kernel(PackPtrs s0, PackPtrs s1, PackPtrs s2, uint4* __restrict__ dst, int P, int d_model,
                                  int d_ffn, size_t n_rows, size_t Kp) {
    constexpr int KB = 4 * V;
    const size_t kblocks = Kp / KB;
    const size_t total = n_rows * kblocks * 4;  // pieces: per row KB/V = 4 per k block
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int i = (int)(idx & 15);
        const int g = (int)((idx >> 4) & 3);
        const size_t tile_id = idx >> 6;
        const size_t kb = tile_id % kblocks, rt = tile_id / kblocks;
        const size_t r = rt * 16 + i;
        const size_t k = kb * KB + (size_t)g * V;
        const uint4* src = nullptr;  // 16-byte piece of a source row, or null for padding
        if (KIND == kPackQkv) {
            const int lm = (int)(r / d_model), o = (int)(r % d_model);
            const int l = lm / 3, m = lm % 3;
            const char* base = m == 0 ? s0.p[l] : (m == 1 ? s1.p[l] : s2.p[l]);
            src = reinterpret_cast<const uint4*>(base) + ((size_t)o * d_model + k) / V;
        } else if (KIND == kPackWo) {
            const int l = (int)(k / d_model), kk = (int)(k % d_model);
            src = reinterpret_cast<const uint4*>(s0.p[l]) + (r * d_model + kk) / V;
        } else if (KIND == kPackGu) {
            const int l = (int)(r / (2 * (size_t)d_ffn));
            const int in = (int)(r % (2 * (size_t)d_ffn));
            const int blk = in / (2 * kGuBlock), w = in % (2 * kGuBlock);
            const int j = blk * kGuBlock + w % kGuBlock;
            const char* base = (w / kGuBlock) ? s1.p[l] : s0.p[l];
            src = reinterpret_cast<const uint4*>(base) + ((size_t)j * d_model + k) / V;
        } else {
            if (k < (size_t)P * d_ffn) {
                const int l = (int)(k / d_ffn), j = (int)(k % d_ffn);
                src = reinterpret_cast<const uint4*>(s0.p[l]) + (r * d_ffn + j) / V;
            }
        }
        dst[idx] = src ? *src : make_uint4(0, 0, 0, 0);
    }
}

// dst[l][:] = gain vector of layer l  (element-wise copy; d_model*esize is a multiple of 16)
__global__ void pack_gain_kernel(PackPtrs g, uint4* dst, int P, int vec_per_row) {
    const int total = P * vec_per_row;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x)
        dst[i] = reinterpret_cast<const uint4*>(g.p[i / vec_per_row])[i % vec_per_row];
}

// table[pos][i] = (cos, sin)(pos * base^(-2i/head_dim)); evaluated in double, rounded once to fp32
__global__ void rope_table_kernel(float2* table, int max_seq, int half, double base) {
    const int total = max_seq * half;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        const int pos = idx / half, i = idx % half;
        const double theta = pow(base, -(double)i / (double)half);
        const double phi = (double)pos * theta;
        table[idx] = make_float2((float)cos(phi), (float)sin(phi));
    }
}

static int grid_for(size_t total, int threads) {
    size_t g = (total + threads - 1) / threads;
    if (g > 65536) g = 65536;
    if (g < 1) g = 1;
    return (int)g;
}

template <int V>
static void pack_all(const cqil_dims& d, int P, const PackArgs& src, char* packed, const cqil_packed_layout& L,
                     hipStream_t st) {
    constexpr int KB = 4 * V;
    const int T = 256, dm = d.d_model, f = d.d_ffn;
    PackPtrs a, b, c;
    for (int l = 0; l < P; ++l) { a.p[l] = (const char*)src.layers[l].wq; b.p[l] = (const char*)src.layers[l].wk; c.p[l] = (const char*)src.layers[l].wv; }
    size_t rows = (size_t)P * 3 * dm, Kp = dm;
    hipLaunchKernelGGL(HIP_KERNEL_NAME(pack_tiled_kernel<kPackQkv, V>), dim3(grid_for(rows * Kp / V, T)), dim3(T), 0, st,
                       a, b, c, (uint4*)(packed + L.wqkv), P, dm, f, rows, Kp);
    for (int l = 0; l < P; ++l) a.p[l] = (const char*)src.layers[l].wo;
    rows = dm; Kp = (size_t)P * dm;
    hipLaunchKernelGGL(HIP_KERNEL_NAME(pack_tiled_kernel<kPackWo, V>), dim3(grid_for(rows * Kp / V, T)), dim3(T), 0, st,
                       a, a, a, (uint4*)(packed + L.wo), P, dm, f, rows, Kp);
    for (int l = 0; l < P; ++l) { a.p[l] = (const char*)src.layers[l].wgate; b.p[l] = (const char*)src.layers[l].wup; }
    rows = (size_t)P * 2 * f; Kp = dm;
    hipLaunchKernelGGL(HIP_KERNEL_NAME(pack_tiled_kernel<kPackGu, V>), dim3(grid_for(rows * Kp / V, T)), dim3(T), 0, st,
                       a, b, b, (uint4*)(packed + L.wgu), P, dm, f, rows, Kp);
    for (int l = 0; l < P; ++l) a.p[l] = (const char*)src.layers[l].wdown;
    rows = dm; Kp = ((size_t)P * f + KB - 1) / KB * KB;
    hipLaunchKernelGGL(HIP_KERNEL_NAME(pack_tiled_kernel<kPackDown, V>), dim3(grid_for(rows * Kp / V, T)), dim3(T), 0,
                       st, a, a, a, (uint4*)(packed + L.wdown), P, dm, f, rows, Kp);
}

hipError_t launch_pack(const cqil_dims& d, int P, const PackArgs& src, char* packed, const cqil_packed_layout& L,
                       hipStream_t st) {
    if (d.dtype == CQIL_BF16) pack_all<8>(d, P, src, packed, L, st);
    else pack_all<4>(d, P, src, packed, L, st);
    const int es = (int)esize(d.dtype);
    const int vpr_dm = d.d_model * es / 16;
    const int T = 256;
    PackPtrs a;
    for (int l = 0; l < P; ++l) a.p[l] = (const char*)src.layers[l].g_attn;
    hipLaunchKernelGGL(pack_gain_kernel, dim3(grid_for((size_t)P * vpr_dm, T)), dim3(T), 0, st, a,
                       (uint4*)(packed + L.g_attn), P, vpr_dm);
    for (int l = 0; l < P; ++l) a.p[l] = (const char*)src.layers[l].g_ffn;
    hipLaunchKernelGGL(pack_gain_kernel, dim3(grid_for((size_t)P * vpr_dm, T)), dim3(T), 0, st, a,
                       (uint4*)(packed + L.g_ffn), P, vpr_dm);
    hipLaunchKernelGGL(rope_table_kernel, dim3(grid_for((size_t)d.max_seq * (d.head_dim / 2), T)), dim3(T), 0, st,
                       (float2*)(packed + L.rope), d.max_seq, d.head_dim / 2, (double)d.rope_base);
    return hipGetLastError();
}

// LoRA merge: W[o][k] += scale * sum_j Bm[o][j] A[j][k], fp32 accumulation, one rounding to the storage type.
// A thread owns kVec consecutive columns of one row (16-byte accesses); r <= kMaxLoraRank.
template <typename T>
__global__ __launch_bounds__(256) void merge_lora_kernel(T* __restrict__ W, const T* __restrict__ A,
                                                         const T* __restrict__ Bm, int n_out, int n_in, int r,
                                                         float scale) {
    constexpr int V = elem<T>::kVec;
    const int cpr = n_in / V;  // chunks per row
    const size_t total = (size_t)n_out * cpr;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t o = i / cpr;
        const int k = (int)(i % cpr) * V;
        float acc[V];
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] = 0.f;
        for (int j = 0; j < r; ++j) {
            const float b = elem<T>::load(Bm + o * r + j);
            float av[V];
            elem<T>::unpack(load16(A + (size_t)j * n_in + k), av);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] = fmaf(b, av[e], acc[e]);
        }
        float wv[V];
        elem<T>::unpack(load16(W + o * n_in + k), wv);
        if constexpr (V == 4) {
            *reinterpret_cast<float4*>(W + o * n_in + k) =
                make_float4(wv[0] + scale * acc[0], wv[1] + scale * acc[1], wv[2] + scale * acc[2], wv[3] + scale * acc[3]);
        } else {
            uint32_t o32[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o32[e] = f32x2_to_bf16x2(wv[2 * e] + scale * acc[2 * e], wv[2 * e + 1] + scale * acc[2 * e + 1]);
            *reinterpret_cast<uint4*>(W + o * n_in + k) = make_uint4(o32[0], o32[1], o32[2], o32[3]);
        }
    }
}

hipError_t launch_merge_lora(void* W, const void* A, const void* Bm, int dtype, int n_out, int n_in, int r, float scale,
                             hipStream_t st) {
    const size_t total = (size_t)n_out * (n_in / (dtype == CQIL_BF16 ? 8 : 4));
    const unsigned grid = (unsigned)((total + 255) / 256 > 65536 ? 65536 : (total + 255) / 256);
    if (dtype == CQIL_BF16)
        hipLaunchKernelGGL(HIP_KERNEL_NAME(merge_lora_kernel<bf16_t>), dim3(grid), dim3(256), 0, st, (bf16_t*)W,
                           (const bf16_t*)A, (const bf16_t*)Bm, n_out, n_in, r, scale);
    else
        hipLaunchKernelGGL(HIP_KERNEL_NAME(merge_lora_kernel<float>), dim3(grid), dim3(256), 0, st, (float*)W,
                           (const float*)A, (const float*)Bm, n_out, n_in, r, scale);
    return hipGetLastError();
}

// Similarity of layer inputs (Sec.3.1).  X [L][M][n]; a workgroup takes one pair (a, b <= a) and one chunk of
// tokens, a wave one token at a time (16-byte loads, fp32 sums); the waves' cosines are added in wave order, the
// chunks by the second kernel in chunk order: deterministic.  part [chunks][L][L].
template <typename T>
__global__ __launch_bounds__(256) void similarity_partial_kernel(const T* __restrict__ X, float* __restrict__ part,
                                                                 int L, int M, int n, int tokens_per_chunk) {
    constexpr int V = elem<T>::kVec;
    __shared__ float wsum[4];
    const int a = blockIdx.x, b = blockIdx.y, chunk = blockIdx.z;
    if (b > a) return;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m0 = chunk * tokens_per_chunk, m1 = min(m0 + tokens_per_chunk, M);
    float acc = 0.f;
    for (int m = m0 + w; m < m1; m += 4) {
        const T* xa = X + ((size_t)a * M + m) * n;
        const T* xb = X + ((size_t)b * M + m) * n;
        float dot = 0.f, na = 0.f, nb = 0.f;
        for (int k = lane * V; k < n; k += 64 * V) {
            float fa[V], fb[V];
            elem<T>::unpack(load16(xa + k), fa);
            elem<T>::unpack(load16(xb + k), fb);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                dot = fmaf(fa[e], fb[e], dot);
                na = fmaf(fa[e], fa[e], na);
                nb = fmaf(fb[e], fb[e], nb);
            }
        }
        dot = wave_sum(dot); na = wave_sum(na); nb = wave_sum(nb);
        if (na > 0.f && nb > 0.f) acc += dot / (sqrtf(na) * sqrtf(nb));
    }
    if (lane == 0) wsum[w] = acc;
    __syncthreads();
    if (threadIdx.x == 0) part[((size_t)chunk * L + a) * L + b] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

__global__ void similarity_reduce_kernel(const float* __restrict__ part, float* __restrict__ sim, int L, int M,
                                         int chunks) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= L * L) return;
    const int a = i / L, b = i % L;
    const int hi = a > b ? a : b, lo = a > b ? b : a;  // only the lower triangle was computed
    float s = 0.f;
    for (int c = 0; c < chunks; ++c) s += part[((size_t)c * L + hi) * L + lo];
    sim[i] = s / (float)M;
}

hipError_t launch_similarity(const void* X, int dtype, int L, int M, int n, float* sim, float* part, int chunks,
                             int tokens_per_chunk, hipStream_t st) {
    const dim3 grid(L, L, chunks);
    if (dtype == CQIL_BF16)
        hipLaunchKernelGGL(HIP_KERNEL_NAME(similarity_partial_kernel<bf16_t>), grid, dim3(256), 0, st, (const bf16_t*)X, part,
                           L, M, n, tokens_per_chunk);
    else
        hipLaunchKernelGGL(HIP_KERNEL_NAME(similarity_partial_kernel<float>), grid, dim3(256), 0, st, (const float*)X, part,
                           L, M, n, tokens_per_chunk);
    hipLaunchKernelGGL(similarity_reduce_kernel, dim3((L * L + 255) / 256), dim3(256), 0, st, part, sim, L, M, chunks);
    return hipGetLastError();
}

// Measurement aid: reads n 16-byte chunks once with the streaming (non-temporal) loads of the decode kernels.  A
// workgroup takes tiles of 256 x 8 consecutive chunks (every load instruction of a wave reads 1 KiB of consecutive
// bytes, eight in flight per thread, the way the decode kernels walk their weight tiles), every index checked against
// n.  The xor of what was read goes to sink[workgroup] so that the loads cannot be dropped.  Gives the rate at which
// this GPU delivers a read-only stream, the ceiling the decode kernels are compared with besides the nameplate.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ buf, size_t n, uint32_t* __restrict__ sink) {
    constexpr int U = 8;
    __shared__ uint32_t ws[4];
    const size_t tile = (size_t)256 * U;
    uint32_t acc = 0;
    for (size_t base = (size_t)blockIdx.x * tile; base < n; base += (size_t)gridDim.x * tile) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = base + (size_t)u * 256 + threadIdx.x;
            v[u] = (i < n) ? load16_stream(buf + i) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc ^= __shfl_xor(acc, off, kWave);
    if ((threadIdx.x & 63) == 0) ws[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = ws[0] ^ ws[1] ^ ws[2] ^ ws[3];
}

hipError_t launch_stream_read(const void* buf, size_t bytes, uint32_t* sink, int workgroups, hipStream_t st) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, st, (const uint4*)buf, bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace cqil
