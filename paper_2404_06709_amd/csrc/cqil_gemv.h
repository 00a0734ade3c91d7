// Streaming matrix-vector building blocks of the decode kernels.
// dot4: row-major matrices (the lm head): a wave owns four rows at a time, each lane reads 16 contiguous bytes of
// each row per step, the input vector sits in LDS as fp32.  tile_strip_dot: the tiled layout of the packed groups.
#pragma once
#include "cqil_dev.h"

namespace cqil {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;

// LDS placement of input element k so that the 16-byte LDS reads of consecutive lanes are consecutive.
// Each lane consumes kVec consecutive elements per step (one 16-byte weight load).
template <int V> __device__ __forceinline__ int xs_index(int k);
template <> __device__ __forceinline__ int xs_index<4>(int k) { return k; }
template <> __device__ __forceinline__ int xs_index<8>(int k) {
    return (k & ~511) + ((k >> 2) & 1) * 256 + ((k & 511) >> 3) * 4 + (k & 3);
}

template <int V> __device__ __forceinline__ void xs_read(const float* xs, int k, float (&out)[V]);
template <> __device__ __forceinline__ void xs_read<4>(const float* xs, int k, float (&out)[4]) {
    const float4 a = *reinterpret_cast<const float4*>(xs + k);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
}
template <> __device__ __forceinline__ void xs_read<8>(const float* xs, int k, float (&out)[8]) {
    const int base = (k & ~511) + ((k & 511) >> 3) * 4;
    const float4 a = *reinterpret_cast<const float4*>(xs + base);
    const float4 b = *reinterpret_cast<const float4*>(xs + base + 256);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
    out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}

// Four dot products of length len (a multiple of kVec) against the LDS-resident input; every lane of the
// calling wave returns the four totals.
template <typename WT>
__device__ __forceinline__ void dot4(const WT* r0, const WT* r1, const WT* r2, const WT* r3, const float* xs,
                                     int len, float (&out)[4]) {
    constexpr int V = elem<WT>::kVec;
    constexpr int step = kWave * V;
    const int lane = threadIdx.x & 63;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    int k = lane * V;
    for (; k + step < len; k += 2 * step) {
        const uint4 w0 = load16_stream(r0 + k), w1 = load16_stream(r1 + k);
        const uint4 w2 = load16_stream(r2 + k), w3 = load16_stream(r3 + k);
        const uint4 v0 = load16_stream(r0 + k + step), v1 = load16_stream(r1 + k + step);
        const uint4 v2 = load16_stream(r2 + k + step), v3 = load16_stream(r3 + k + step);
        float x[V], f[V];
        xs_read<V>(xs, k, x);
        elem<WT>::unpack(w0, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[0] = fmaf(f[j], x[j], acc[0]);
        elem<WT>::unpack(w1, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[1] = fmaf(f[j], x[j], acc[1]);
        elem<WT>::unpack(w2, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[2] = fmaf(f[j], x[j], acc[2]);
        elem<WT>::unpack(w3, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[3] = fmaf(f[j], x[j], acc[3]);
        xs_read<V>(xs, k + step, x);
        elem<WT>::unpack(v0, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[0] = fmaf(f[j], x[j], acc[0]);
        elem<WT>::unpack(v1, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[1] = fmaf(f[j], x[j], acc[1]);
        elem<WT>::unpack(v2, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[2] = fmaf(f[j], x[j], acc[2]);
        elem<WT>::unpack(v3, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[3] = fmaf(f[j], x[j], acc[3]);
    }
    if (k < len) {
        const uint4 w0 = load16_stream(r0 + k), w1 = load16_stream(r1 + k);
        const uint4 w2 = load16_stream(r2 + k), w3 = load16_stream(r3 + k);
        float x[V], f[V];
        xs_read<V>(xs, k, x);
        elem<WT>::unpack(w0, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[0] = fmaf(f[j], x[j], acc[0]);
        elem<WT>::unpack(w1, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[1] = fmaf(f[j], x[j], acc[1]);
        elem<WT>::unpack(w2, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[2] = fmaf(f[j], x[j], acc[2]);
        elem<WT>::unpack(w3, f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[3] = fmaf(f[j], x[j], acc[3]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) out[r] = wave_sum(acc[r]);
}

__device__ __forceinline__ int xs_words(int len) { return (len + 511) & ~511; }

// ---------------------------------------------------------------------------------------------------------
// Streaming block over the tiled weight layout (tile<> in cqil_dev.h).  A wave walks one 16-row strip: every
// 16-byte load of the wave reads one whole 1 KiB tile (fully contiguous), U tiles in flight; lane i + 16 g holds
// kVec columns (k group g) of row i and multiplies them with the matching input values, which sit in LDS as fp32
// in natural order (the 16 lanes of a k group read the same address: a broadcast).  The four k groups of a row
// are added with two cross-lane steps; every lane returns the dot product of row (lane % 16) over the n_kb tiles.
//   strip[s]  first tile of the range of strip s (NS strips advance together, NS * U tiles in flight)
//   xs        input values of the first column of the range
// ---------------------------------------------------------------------------------------------------------
// tile_strips_prefetch issues the loads of the first U tiles of every strip (n_kb <= 0: none) and
// tile_strips_dot takes them as its first batch: a kernel calls the former before it stages its input vector in
// LDS (norm, barriers), so that the weight stream starts with the kernel and not after that prologue.
template <typename T, int NS, int U>
__device__ __forceinline__ void tile_strips_prefetch(const T* const (&strip)[NS], int n_kb, uint4 (&w)[NS][U]) {
    constexpr int V = tile<T>::V, TE = tile<T>::kElems;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int u = 0; u < U; ++u)
            w[s][u] = (u < n_kb) ? load16_stream(strip[s] + (size_t)u * TE + lane * V) : make_uint4(0, 0, 0, 0);
}

template <typename T, int NS, int U>
__device__ __forceinline__ void tile_strips_dot(const T* const (&strip)[NS], int n_kb, const float* xs,
                                                uint4 (&w)[NS][U], float (&out)[NS]) {
    constexpr int V = tile<T>::V, KB = tile<T>::KB, TE = tile<T>::kElems;
    const int lane = threadIdx.x & 63;
    const float* xg = xs + (lane >> 4) * V;
    float acc[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) acc[s] = 0.f;
    for (int kb = 0; kb < n_kb; kb += U) {
        // NS * U tiles in flight; the conditions are wave-uniform (ragged end of the range)
        if (kb > 0) {
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (kb + u < n_kb) w[s][u] = load16_stream(strip[s] + (size_t)(kb + u) * TE + lane * V);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kb + u < n_kb) {
                float x[V];
                const float* xp = xg + (kb + u) * KB;
#pragma unroll
                for (int e = 0; e < V; e += 4) {
                    const float4 xv = *reinterpret_cast<const float4*>(xp + e);
                    x[e] = xv.x; x[e + 1] = xv.y; x[e + 2] = xv.z; x[e + 3] = xv.w;
                }
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    float f[V];
                    elem<T>::unpack(w[s][u], f);
#pragma unroll
                    for (int e = 0; e < V; ++e) acc[s] = fmaf(f[e], x[e], acc[s]);
                }
            }
        }
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        acc[s] += __shfl_xor(acc[s], 16, kWave);
        acc[s] += __shfl_xor(acc[s], 32, kWave);
        out[s] = acc[s];
    }
}

}  // namespace cqil
