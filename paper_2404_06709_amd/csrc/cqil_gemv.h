// Streaming matrix-vector building block shared by the decode kernels: a wave owns four weight rows at a
// time, each lane reads 16 contiguous bytes of each row per step, the input vector sits in LDS as fp32.
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
// Software-pipelined version of the same block.  A wave walks a sequence of row groups (four rows each) and,
// inside a group, tiles of two 16-byte steps; the loads of the NEXT tile (of this group or of the wave's next
// group) are issued before the current tile is consumed, so a wave always has 8 to 16 loads in flight.
//   rows(g, r)  fills the four row pointers of group g
//   done(g, s)  receives the four totals of group g (in every lane)
// Groups g = g_begin, g_begin + g_stride, ... < g_end.
// ---------------------------------------------------------------------------------------------------------
template <typename WT>
struct Tile2 {
    uint4 w[8];
};

template <typename WT>
__device__ __forceinline__ void tile_load(Tile2<WT>& t, const WT* const (&r)[4], int k, int len) {
    constexpr int step = kWave * elem<WT>::kVec;
    const bool second = k + step < len;
#pragma unroll
    for (int j = 0; j < 4; ++j) t.w[j] = load16_stream(r[j] + k);
#pragma unroll
    for (int j = 0; j < 4; ++j) t.w[4 + j] = second ? load16_stream(r[j] + k + step) : make_uint4(0, 0, 0, 0);
}

template <typename WT>
__device__ __forceinline__ void tile_fma(const Tile2<WT>& t, const float* xs, int k, int len, float (&acc)[4]) {
    constexpr int V = elem<WT>::kVec;
    constexpr int step = kWave * V;
    float x[V], f[V];
    xs_read<V>(xs, k, x);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        elem<WT>::unpack(t.w[j], f);
#pragma unroll
        for (int e = 0; e < V; ++e) acc[j] = fmaf(f[e], x[e], acc[j]);
    }
    if (k + step < len) {
        xs_read<V>(xs, k + step, x);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            elem<WT>::unpack(t.w[4 + j], f);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[j] = fmaf(f[e], x[e], acc[j]);
        }
    }
}

template <typename WT, typename RowFn, typename DoneFn>
__device__ __forceinline__ void stream_groups(int g_begin, int g_end, int g_stride, int len, const float* xs,
                                              RowFn rows, DoneFn done) {
    constexpr int V = elem<WT>::kVec;
    constexpr int step = kWave * V;
    const int lane = threadIdx.x & 63;
    const int k_lane = lane * V;
    if (g_begin >= g_end) return;
    // lanes whose first element lies beyond len idle for the whole call (len < 64*V only in tiny shapes)
    const bool lane_on = k_lane < len;
    const WT* r[4];
    rows(g_begin, r);
    Tile2<WT> cur;
    if (lane_on) tile_load<WT>(cur, r, k_lane, len);
    for (int g = g_begin; g < g_end; g += g_stride) {
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        const WT* rn[4];
        const bool more_groups = g + g_stride < g_end;
        if (more_groups) rows(g + g_stride, rn);
        for (int k = k_lane; k < len; k += 2 * step) {
            Tile2<WT> nxt;
            const int kn = k + 2 * step;
            if (kn < len) tile_load<WT>(nxt, r, kn, len);
            else if (more_groups) tile_load<WT>(nxt, rn, k_lane, len);
            tile_fma<WT>(cur, xs, k, len, acc);
            cur = nxt;
        }
        float s[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) s[j] = wave_sum(acc[j]);
        done(g, s);
#pragma unroll
        for (int j = 0; j < 4; ++j) r[j] = rn[j];
    }
}


// One row at a time: up to NCH 16-byte steps of ONE row in flight per lane (a wave requests NCH KiB of
// contiguous memory back to back), then the next row.
template <typename WT, int NCH>
__device__ __forceinline__ float row_dot(const WT* r, const float* xs, int len) {
    constexpr int V = elem<WT>::kVec;
    constexpr int step = kWave * V;
    const int lane = threadIdx.x & 63;
    float acc = 0.f;
    for (int k0 = lane * V; k0 < len; k0 += NCH * step) {
        uint4 w[NCH];
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int k = k0 + c * step;
            w[c] = k < len ? load16_stream(r + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int k = k0 + c * step;
            if (k < len) {
                float x[V], f[V];
                xs_read<V>(xs, k, x);
                elem<WT>::unpack(w[c], f);
#pragma unroll
                for (int e = 0; e < V; ++e) acc = fmaf(f[e], x[e], acc);
            }
        }
    }
    return wave_sum(acc);
}

template <typename WT, int NCH, typename RowFn, typename DoneFn>
__device__ __forceinline__ void stream_groups_rowwise(int g_begin, int g_end, int g_stride, int len, const float* xs,
                                                      RowFn rows, DoneFn done) {
    for (int g = g_begin; g < g_end; g += g_stride) {
        const WT* r[4];
        rows(g, r);
        float s[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) s[j] = row_dot<WT, NCH>(r[j], xs, len);
        done(g, s);
    }
}

// Same interface without the cross-tile prefetch (one dot4 per group).
template <typename WT, typename RowFn, typename DoneFn>
__device__ __forceinline__ void stream_groups_simple(int g_begin, int g_end, int g_stride, int len, const float* xs,
                                                     RowFn rows, DoneFn done) {
    for (int g = g_begin; g < g_end; g += g_stride) {
        const WT* r[4];
        rows(g, r);
        float s[4];
        dot4<WT>(r[0], r[1], r[2], r[3], xs, len, s);
        done(g, s);
    }
}

template <typename WT, int PIPE, typename RowFn, typename DoneFn>
__device__ __forceinline__ void stream_rows(int g_begin, int g_end, int g_stride, int len, const float* xs, RowFn rows,
                                            DoneFn done) {
    if constexpr (PIPE == 1) stream_groups<WT>(g_begin, g_end, g_stride, len, xs, rows, done);
    else if constexpr (PIPE == 2) stream_groups_rowwise<WT, 16>(g_begin, g_end, g_stride, len, xs, rows, done);
    else if constexpr (PIPE == 3) stream_groups_rowwise<WT, 8>(g_begin, g_end, g_stride, len, xs, rows, done);
    else stream_groups_simple<WT>(g_begin, g_end, g_stride, len, xs, rows, done);
}

}  // namespace cqil
