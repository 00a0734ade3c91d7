// Streaming matrix-vector building block shared by the decode kernels: a wave owns four weight rows at a
// time, each lane reads 16 contiguous bytes of each row per step, the input vector sits in LDS as fp32.
#pragma once
#include "cqil_dev.h"

namespace cqil {

constexpr int kThreads = 256;
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

}  // namespace cqil
