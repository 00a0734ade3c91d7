// Device-side helpers shared by the CQIL kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cqil {

typedef uint16_t bf16_t;  // raw bf16 bit pattern

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even; NaN stays NaN.  The casts compile to v_cvt_pk_bf16_f32 on gfx950.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values -> one dword (a in the low half)
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float a, float b) {
    typedef float cvt_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 cvt_bf16x2 __attribute__((ext_vector_type(2)));
    const cvt_f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, cvt_bf16x2));
}

template <typename T> struct elem;
template <> struct elem<float> {
    static constexpr int kVec = 4;  // elements per 16-byte load
    __device__ static __forceinline__ float load(const float* p) { return *p; }
    __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
    // 16-byte vector -> kVec floats
    __device__ static __forceinline__ void unpack(const uint4& v, float (&out)[4]) {
        out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
        out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
    }
};
template <> struct elem<bf16_t> {
    static constexpr int kVec = 8;
    __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
    __device__ static __forceinline__ void unpack(const uint4& v, float (&out)[8]) {
        out[0] = __uint_as_float(v.x << 16); out[1] = __uint_as_float(v.x & 0xffff0000u);
        out[2] = __uint_as_float(v.y << 16); out[3] = __uint_as_float(v.y & 0xffff0000u);
        out[4] = __uint_as_float(v.z << 16); out[5] = __uint_as_float(v.z & 0xffff0000u);
        out[6] = __uint_as_float(v.w << 16); out[7] = __uint_as_float(v.w & 0xffff0000u);
    }
};

// ---------------------------------------------------------------------------------------------------------
// Tiled weight layout.  A logical matrix W[R][K] (R a multiple of 16, K padded to Kp, a multiple of the k block
// KB = 4 * kVec) is stored as 1 KiB tiles of 16 rows x KB columns; the tiles of one 16-row strip follow each other
// along k.  Inside a tile the order is [g = (k % KB) / kVec][i = r % 16][e = k % kVec], i.e. the 16-byte piece of
// lane i + 16 g of a wave: one wave-wide 16-byte load reads one whole tile, fully contiguous, and the piece a
// lane receives is exactly its fragment of the A operand of v_mfma_f32_16x16x32_bf16 (row i, k group g).
// ---------------------------------------------------------------------------------------------------------
template <typename T> struct tile {
    static constexpr int V = 16 / (int)sizeof(T);  // elements per 16-byte piece
    static constexpr int KB = 4 * V;               // columns per tile (32 for bf16, 16 for fp32)
    static constexpr int kElems = 16 * KB;         // elements per tile (1 KiB)
    __host__ __device__ static inline size_t offset(size_t r, size_t k, size_t Kp) {
        return ((r >> 4) * (Kp / KB) + k / KB) * kElems + ((k % KB) / V) * (16 * V) + (r & 15) * V + (k % V);
    }
};

// 16-byte global load of streamed (read-once) data
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const void* p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 load16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

// Sum over aligned groups of G consecutive lanes (G = 2 .. 64, a power of two); every lane returns its group's total.
// Up to 16 lanes the partner values come through the ALU's data-parallel lane permutes (within quads: lane ^ 1,
// lane ^ 2; then the mirror of each half row and of each row of 16), not through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int G>
__device__ __forceinline__ float lane_group_sum(float v) {
    if (G >= 2) v += dpp_move<0xB1>(v);    // quad_perm [1, 0, 3, 2]
    if (G >= 4) v += dpp_move<0x4E>(v);    // quad_perm [2, 3, 0, 1]
    if (G >= 8) v += dpp_move<0x141>(v);   // row_half_mirror
    if (G >= 16) v += dpp_move<0x140>(v);  // row_mirror
    if (G >= 32) v += __shfl_xor(v, 16, kWave);
    if (G >= 64) v += __shfl_xor(v, 32, kWave);
    return v;
}

// Sum over the 64 lanes of a wave; every lane returns the total.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// Sum over all threads of a block (blockDim.x a multiple of 64, at most 1024); scratch holds >= 16 floats.
// Every thread returns the total.  Contains two barriers.
__device__ __forceinline__ float block_sum(float v, float* scratch) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += scratch[i];
    return t;
}

}  // namespace cqil
