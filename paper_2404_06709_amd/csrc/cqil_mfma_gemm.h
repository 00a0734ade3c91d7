// bf16 matrix-core GEMM of the token-parallel (prefill) path:  C[m][n] = sum_k A[m][k] * W[n][k]  (+ R[m][n]).
//
// A: activations, row-major [M][lda] bf16.  W: a packed weight matrix in the tiled layout (tile<> in cqil_dev.h),
// padded width Kp; a group z (blockIdx.z) addresses a row band (N-concatenation) or a column band
// (K-concatenation) of it.  C: row-major, bf16 or fp32; fp32 accumulation.
//
// Workgroup tile 256 tokens x 256 weight rows x 64 columns, 8 waves as 2 (tokens) x 4 (weight rows); a wave owns
// 128 tokens x 64 weight rows = 8 x 4 tiles of v_mfma_f32_16x16x32_bf16 (128 accumulator registers).  The weight
// rows are the instruction's A operand, the tokens its B operand, so a lane ends up with 4 consecutive weight
// rows of one token: 4 consecutive elements of a C row.
// Both operands are staged in LDS as 1 KiB tiles in operand order, so every fragment read is one contiguous
// 16-byte-per-lane read without bank conflicts: weight tiles are copied verbatim (they are stored that way);
// activation rows are re-tiled on the way in, with the 16-byte pieces of a tile rotated by 4 g + 2 kt so that
// the eight pieces of one 128-byte row segment, which eight neighbouring threads write, fall into different banks.
// Two LDS stages: the global loads of step i+1 are in flight while step i is multiplied.
#pragma once
#include "cqil_dev.h"

namespace cqil {

typedef __bf16 gemm_bf16x8 __attribute__((ext_vector_type(8)));
typedef float gemm_f32x4 __attribute__((ext_vector_type(4)));

constexpr int kGemmBM = 256, kGemmBN = 256, kGemmBK = 64, kGemmThreads = 512;
constexpr int kGemmStageElems = (kGemmBM + kGemmBN) * kGemmBK;         // bf16 elements per stage
constexpr size_t kGemmLdsBytes = 2 * (size_t)kGemmStageElems * 2;      // two stages

__device__ __forceinline__ void gemm_store4(bf16_t* p, const float (&v)[4]) {
    uint2 o;
    o.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
    o.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
    *reinterpret_cast<uint2*>(p) = o;
}
__device__ __forceinline__ void gemm_store4(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}

// N, K: logical sizes of this group's product; N % 4 == 0.  n_strip0 / k_tile0: first 16-row strip / first
// 32-column tile of the group inside W.  R (ADD_R): fp32 [M][N] added to the result.
template <typename CT, bool ADD_R>
__global__ __launch_bounds__(kGemmThreads) void gemm_mfma_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, CT* __restrict__ C, const float* __restrict__ R, int M,
    int N, int K, size_t lda, size_t Kp, size_t ldc, size_t sA, size_t strip_step, size_t ktile_step, size_t sC) {
    extern __shared__ __align__(16) unsigned char gemm_smem[];
    bf16_t* lds = reinterpret_cast<bf16_t*>(gemm_smem);
    constexpr int TE = 512;  // elements per tile
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int wm = w >> 2, wn = w & 3;
    const int z = blockIdx.z;
    A += (size_t)z * sA;
    C += (size_t)z * sC;
    const size_t n_strip0 = (size_t)z * strip_step, k_tile0 = (size_t)z * ktile_step;
    const int m0 = blockIdx.y * kGemmBM, n0 = blockIdx.x * kGemmBN;
    const size_t w_tiles_per_strip = Kp / 32;
    const int n_strips = N / 16 + ((N % 16) ? 1 : 0);   // strips of this group that exist (N % 16 == 0 in practice)
    const int n_ktiles = (K + 31) / 32;
    const int n_steps = (n_ktiles + 1) / 2;

    // ---- global -> register staging of one step (4 weight pieces, 4 activation pieces per thread)
    uint4 wreg[4], areg[4];
    auto load_step = [&](int step) {
        const int kt0 = 2 * step;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int tile_idx = w + 8 * q;              // 0..31 = strip_local * 2 + kt
            const int strip = n0 / 16 + (tile_idx >> 1);
            const int kt = kt0 + (tile_idx & 1);
            wreg[q] = (strip < n_strips && kt < n_ktiles)
                          ? *reinterpret_cast<const uint4*>(W + ((n_strip0 + strip) * w_tiles_per_strip + k_tile0 + kt) * TE + lane * 8)
                          : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = (tid >> 3) + 64 * q;         // 0..255
            const int c = tid & 7;                       // 16-byte piece along k
            const int m = m0 + row, k = 64 * step + 8 * c;
            areg[q] = (m < M && k < K) ? *reinterpret_cast<const uint4*>(A + (size_t)m * lda + k) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_step = [&](int buf) {
        bf16_t* ws = lds + (size_t)buf * kGemmStageElems;
        bf16_t* as = ws + kGemmBN * kGemmBK;
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<uint4*>(ws + (w + 8 * q) * TE + lane * 8) = wreg[q];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = (tid >> 3) + 64 * q, c = tid & 7;
            const int ts = row >> 4, j = row & 15, kt = c >> 2, g = c & 3;
            const int pos = g * 16 + ((j + 4 * g + 2 * kt) & 15);
            *reinterpret_cast<uint4*>(as + (ts * 2 + kt) * TE + pos * 8) = areg[q];
        }
    };

    gemm_f32x4 acc[8][4];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[t][s] = gemm_f32x4{0.f, 0.f, 0.f, 0.f};

    const int j = lane & 15, g = lane >> 4;
    load_step(0);
    store_step(0);
    __syncthreads();
    for (int step = 0; step < n_steps; ++step) {
        const int buf = step & 1;
        if (step + 1 < n_steps) load_step(step + 1);
        const bf16_t* ws = lds + (size_t)buf * kGemmStageElems;
        const bf16_t* as = ws + kGemmBN * kGemmBK;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            uint4 wf[4], af[8];
#pragma unroll
            for (int s = 0; s < 4; ++s) wf[s] = *reinterpret_cast<const uint4*>(ws + ((4 * wn + s) * 2 + kt) * TE + lane * 8);
            const int pos = g * 16 + ((j + 4 * g + 2 * kt) & 15);
#pragma unroll
            for (int t = 0; t < 8; ++t) af[t] = *reinterpret_cast<const uint4*>(as + ((8 * wm + t) * 2 + kt) * TE + pos * 8);
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc[t][s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(gemm_bf16x8, wf[s]),
                                                                        __builtin_bit_cast(gemm_bf16x8, af[t]), acc[t][s], 0, 0, 0);
        }
        if (step + 1 < n_steps) store_step(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane (j, g) holds weight rows 4g .. 4g+3 of token j of every 16x16 tile
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int m = m0 + 128 * wm + 16 * t + j;
        if (m >= M) continue;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int n = n0 + 64 * wn + 16 * s + 4 * g;
            if (n >= N) continue;
            float v[4] = {acc[t][s][0], acc[t][s][1], acc[t][s][2], acc[t][s][3]};
            if (ADD_R) {
                const float4 r = *reinterpret_cast<const float4*>(R + (size_t)m * N + n);
                v[0] += r.x; v[1] += r.y; v[2] += r.z; v[3] += r.w;
            }
            gemm_store4(C + (size_t)m * ldc + n, v);
        }
    }
}

// Same argument convention as the plain kernel of the token-parallel path: n_step / k_step are the group strides
// in weight rows / columns (multiples of 16 / 32).
template <typename CT, bool ADD_R>
static hipError_t gemm_mfma(const bf16_t* A, const bf16_t* W, CT* C, const float* R, int M, int N, int K, size_t lda,
                            size_t Kp, size_t ldc, int groups, size_t sA, size_t n_step, size_t k_step, size_t sC,
                            hipStream_t st) {
    static bool allowed = false;
    if (!allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_mfma_kernel<CT, ADD_R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmLdsBytes);
        if (e != hipSuccess) return e;
        allowed = true;
    }
    dim3 grid((N + kGemmBN - 1) / kGemmBN, (M + kGemmBM - 1) / kGemmBM, groups);
    hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_mfma_kernel<CT, ADD_R>), grid, dim3(kGemmThreads), kGemmLdsBytes, st, A, W, C,
                       R, M, N, K, lda, Kp, ldc, sA, n_step / 16, k_step / 32, sC);
    return hipSuccess;
}

}  // namespace cqil
