// Decode step of one CQIL group for a few token rows at once (2 <= M = B*T <= 8, bf16): the same six kernels
// as the single-token path, with the projections on the matrix cores.
//
// The step stays HBM-bound (every weight byte is still read once), but M dot products per weight would saturate
// the vector ALUs, so each wave multiplies 16-row weight strips by the M token columns with
// v_mfma_f32_16x16x32_bf16.  The packed weights are already stored as the instruction's A operand: one
// wave-wide 16-byte load reads one contiguous 1 KiB tile and lane i + 16 g receives row i, k group g (tile<> in
// cqil_dev.h).  The activations are the B operand, read from LDS (bf16, one row per token; columns beyond M are
// zero).
//   D[i][j] lands in lane j + 16*(i/4), register i%4: a lane holds four consecutive weight rows of one token, so
//   the rotary pairs (strips t and t + head_dim/32) and the gate/up pairs (the packed 16-row blocks) meet in one lane.
#include "cqil_attn.h"
#include "cqil_dev.h"
#include "cqil_internal.h"

namespace cqil {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kSkPad = 32;  // bf16 elements of padding per LDS activation row (64 bytes: spreads the rows over banks)

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4& v) { return __builtin_bit_cast(bf16x8_t, v); }

// NT strips of 16 weight rows times the token columns over n_kb tiles (32 columns each), U tiles of every strip in
// flight.
//   strip[t]  first tile of the range of strip t
//   xrow      this lane's token row in LDS at the first column of the range plus 8*(lane/16); tok_on false ->
//             column of zeros (token index >= M)
template <int NT, int U>
__device__ __forceinline__ void mfma_strips(const bf16_t* const (&strip)[NT], int n_kb, const bf16_t* xrow, bool tok_on,
                                            f32x4_t (&acc)[NT]) {
    constexpr int TE = tile<bf16_t>::kElems, KB = tile<bf16_t>::KB;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    const int lane = threadIdx.x & 63;
    for (int kb = 0; kb < n_kb; kb += U) {
        uint4 a[NT][U], b[U];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int u = 0; u < U; ++u)
                a[t][u] = (kb + u < n_kb) ? load16_stream(strip[t] + (size_t)(kb + u) * TE + lane * 8) : zero;
#pragma unroll
        for (int u = 0; u < U; ++u)
            b[u] = (tok_on && kb + u < n_kb) ? *reinterpret_cast<const uint4*>(xrow + (kb + u) * KB) : zero;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a[t][u]), as_bf16x8(b[u]), acc[t], 0, 0, 0);
    }
}

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) { elem<bf16_t>::unpack(v, f); }
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
    uint4 v;
    v.x = (uint32_t)f32_to_bf16(f[0]) | ((uint32_t)f32_to_bf16(f[1]) << 16);
    v.y = (uint32_t)f32_to_bf16(f[2]) | ((uint32_t)f32_to_bf16(f[3]) << 16);
    v.z = (uint32_t)f32_to_bf16(f[4]) | ((uint32_t)f32_to_bf16(f[5]) << 16);
    v.w = (uint32_t)f32_to_bf16(f[6]) | ((uint32_t)f32_to_bf16(f[7]) << 16);
    return v;
}
__device__ __forceinline__ void load8_f32(const float* p, float (&f)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}

// Builds the LDS activation rows: a wave takes whole token rows (w, w + NW, ...), 8 elements per lane and step
// with 16-byte loads.  With NORM the row is RMS-normalised and multiplied by the gain (two passes over the row:
// statistic, then values).  load8(j, v, out) supplies elements 8v .. 8v+7 of token row j.  Ends with a barrier.
template <bool NORM, typename Load8>
__device__ __forceinline__ void fill_rows(bf16_t* xs, int kpad, int M, int d_model, float eps, const bf16_t* gain,
                                          int n_waves, Load8 load8) {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nvec = d_model / 8;
    for (int j = w; j < M; j += n_waves) {
        float r = 1.0f;
        if (NORM) {
            float ss = 0.f;
#pragma unroll 4
            for (int v = lane; v < nvec; v += kWave) {
                float h[8];
                load8(j, v, h);
#pragma unroll
                for (int e = 0; e < 8; ++e) ss = fmaf(h[e], h[e], ss);
            }
            ss = wave_sum(ss);
            r = 1.0f / sqrtf(ss / (float)d_model + eps);
        }
#pragma unroll 4
        for (int v = lane; v < nvec; v += kWave) {
            float h[8];
            load8(j, v, h);
            if (NORM) {
                float g[8];
                unpack8(*reinterpret_cast<const uint4*>(gain + 8 * v), g);
#pragma unroll
                for (int e = 0; e < 8; ++e) h[e] = h[e] * r * g[e];
            }
            *reinterpret_cast<uint4*>(xs + (size_t)j * kpad + 8 * v) = pack8(h);
        }
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------------------
// 1. RMSNorm + QKV projection + rotary embedding + KV append.  grid = (pair blocks, P), NW waves; a wave owns the
//    two 16-row tiles that hold the two halves of 16 rotary pairs of one head.
// ---------------------------------------------------------------------------------------------------------
template <int NW>
__global__ __launch_bounds__(NW * 64) void qkv_skinny_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ wqkv, const bf16_t* __restrict__ g_attn,
    const float2* __restrict__ rope, const int32_t* __restrict__ kv_len, bf16_t* __restrict__ kc,
    bf16_t* __restrict__ vc, float* __restrict__ q_out, int M, int T_new, int d_model, int n_heads, int d_k,
    int max_seq, int b_max, float eps) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* xs = reinterpret_cast<bf16_t*>(smem_raw);
    const int kpad = d_model + kSkPad;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int l = blockIdx.y;
    fill_rows<true>(xs, kpad, M, d_model, eps, g_attn + (size_t)l * d_model, NW, [&](int j, int v, float (&h)[8]) {
        unpack8(*reinterpret_cast<const uint4*>(x + (size_t)j * d_model + 8 * v), h);
    });

    const int half = d_k >> 1;
    const int pairs_per_head = half / 16;
    const int pairs_per_layer = 3 * n_heads * pairs_per_head;
    const int pi = blockIdx.x * NW + w;
    if (pi >= pairs_per_layer) return;
    const int tp = pi % pairs_per_head;
    const int hu = pi / pairs_per_head;
    const int h = hu % n_heads, m3 = hu / n_heads;  // 0,1,2 = q,k,v
    const int i = lane & 15, gq = lane >> 4;
    const int nkb = d_model / 32;
    const size_t strip_a = ((size_t)(l * 3 + m3) * d_model + (size_t)h * d_k + 16 * tp) / 16;
    const bf16_t* strip[2] = {wqkv + strip_a * nkb * tile<bf16_t>::kElems,
                              wqkv + (strip_a + half / 16) * nkb * tile<bf16_t>::kElems};
    f32x4_t acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    const int j = i;  // token column of this lane
    mfma_strips<2, 8>(strip, nkb, xs + (size_t)j * kpad + 8 * gq, j < M, acc);

    if (j < M) {
        const int b = j / T_new, t = j % T_new;
        const int pos = kv_len[b] + t;
        if (pos >= 0 && pos < max_seq) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = 16 * tp + 4 * gq + r;  // rotary pair (e, e + half)
                const float y1 = acc[0][r], y2 = acc[1][r];
                if (m3 == 2) {
                    bf16_t* dst = vc + ((((size_t)l * b_max + b) * n_heads + h) * max_seq + pos) * d_k;
                    dst[e] = f32_to_bf16(y1);
                    dst[e + half] = f32_to_bf16(y2);
                } else {
                    const float2 cs = rope[(size_t)pos * half + e];
                    const float ra = y1 * cs.x - y2 * cs.y, rb = y2 * cs.x + y1 * cs.y;
                    if (m3 == 0) {
                        float* dst = q_out + ((size_t)l * M + j) * d_model + (size_t)h * d_k;
                        dst[e] = ra;
                        dst[e + half] = rb;
                    } else {
                        bf16_t* dst = kc + ((((size_t)l * b_max + b) * n_heads + h) * max_seq + pos) * d_k;
                        dst[e] = f32_to_bf16(ra);
                        dst[e + half] = f32_to_bf16(rb);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// 3. Output projection per layer: a_l = Wo_l ctx_l.  grid = (tile blocks, P); a wave owns one 16-row tile.
// ---------------------------------------------------------------------------------------------------------
template <int NW>
__global__ __launch_bounds__(NW * 64) void oproj_skinny_kernel(const float* __restrict__ ctx,
                                                               const bf16_t* __restrict__ wo, float* __restrict__ a,
                                                               int P, int M, int d_model) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* xs = reinterpret_cast<bf16_t*>(smem_raw);
    const int kpad = d_model + kSkPad;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int l = blockIdx.y;
    const float* c = ctx + (size_t)l * M * d_model;
    fill_rows<false>(xs, kpad, M, d_model, 0.f, nullptr, NW,
                     [&](int j, int v, float (&h)[8]) { load8_f32(c + (size_t)j * d_model + 8 * v, h); });
    const int ti = blockIdx.x * NW + w;
    if (ti >= d_model / 16) return;
    const int i = lane & 15, gq = lane >> 4;
    const int nkb = d_model / 32;  // tiles of one layer; a strip holds the P layers' tiles one after the other
    const bf16_t* strip[1] = {wo + ((size_t)ti * P * nkb + (size_t)l * nkb) * tile<bf16_t>::kElems};
    f32x4_t acc[1] = {{0.f, 0.f, 0.f, 0.f}};
    mfma_strips<1, 8>(strip, nkb, xs + (size_t)i * kpad + 8 * gq, i < M, acc);
    if (i < M) {
        float* dst = a + ((size_t)l * M + i) * d_model + 16 * ti + 4 * gq;
        *reinterpret_cast<float4*>(dst) = make_float4(acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
    }
}

// ---------------------------------------------------------------------------------------------------------
// 4. Bypass window (Eq.4) + FFN RMSNorm + gate/up projection + SwiGLU.  grid = (j blocks, P); a wave owns one
//    packed block: 16 gate rows and the matching 16 up rows.
// ---------------------------------------------------------------------------------------------------------
template <int NW>
__global__ __launch_bounds__(NW * 64) void gateup_skinny_kernel(const bf16_t* __restrict__ x,
                                                                const float* __restrict__ a,
                                                                const bf16_t* __restrict__ wgu,
                                                                const bf16_t* __restrict__ g_ffn,
                                                                bf16_t* __restrict__ u, int P, int bypass_d, int M,
                                                                int d_model, int d_ffn, float eps) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* xs = reinterpret_cast<bf16_t*>(smem_raw);
    const int kpad = d_model + kSkPad;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int l = blockIdx.y;
    const int jlo = max(0, l - bypass_d);
    const size_t Md = (size_t)M * d_model;
    fill_rows<true>(xs, kpad, M, d_model, eps, g_ffn + (size_t)l * d_model, NW, [&](int j, int v, float (&h)[8]) {
        const size_t idx = (size_t)j * d_model + 8 * v;
        unpack8(*reinterpret_cast<const uint4*>(x + idx), h);
        for (int jj = jlo; jj <= l; ++jj) {
            float t[8];
            load8_f32(a + (size_t)jj * Md + idx, t);
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] += t[e];
        }
    });
    const int jb = blockIdx.x * NW + w;  // block of 16 feed-forward units
    if (jb >= d_ffn / kGuBlock) return;
    const int i = lane & 15, gq = lane >> 4;
    const int nkb = d_model / 32;
    const size_t strip_g = (size_t)l * 2 * d_ffn / 16 + 2 * (size_t)jb;  // gate strip; the up strip follows it
    const bf16_t* strip[2] = {wgu + strip_g * nkb * tile<bf16_t>::kElems, wgu + (strip_g + 1) * nkb * tile<bf16_t>::kElems};
    f32x4_t acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    mfma_strips<2, 8>(strip, nkb, xs + (size_t)i * kpad + 8 * gq, i < M, acc);
    if (i < M) {
        bf16_t* dst = u + (size_t)i * P * d_ffn + (size_t)l * d_ffn + jb * kGuBlock + 4 * gq;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float gt = acc[0][r];
            dst[r] = f32_to_bf16(gt / (1.0f + expf(-gt)) * acc[1][r]);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// 5. Down projection over the K-concatenated Wdown, split along K.  grid = (tile blocks, K slices); partial sums
//    [slice][M][d_model] are added by merge_kernel in slice order.
// ---------------------------------------------------------------------------------------------------------
template <int NW>
__global__ __launch_bounds__(NW * 64) void down_skinny_kernel(const bf16_t* __restrict__ u,
                                                              const bf16_t* __restrict__ wdown,
                                                              float* __restrict__ part, int M, int d_model, int K,
                                                              int slice_len) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* xs = reinterpret_cast<bf16_t*>(smem_raw);
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int slice = blockIdx.y;
    const int k0 = slice * slice_len;
    const int Kp = (K + 31) / 32 * 32;        // the packed matrix is zero-padded to whole tiles
    const int len = min(slice_len, Kp - k0);  // multiple of 32
    const int kpad = slice_len + kSkPad;
    const int vec = len / 8;  // 16-byte vectors per token row of this slice
    for (int idx = tid; idx < M * vec; idx += NW * 64) {
        const int j = idx / vec, v = idx - j * vec;
        const int k = k0 + 8 * v;
        *reinterpret_cast<uint4*>(xs + (size_t)j * kpad + 8 * v) =
            k < K ? *reinterpret_cast<const uint4*>(u + (size_t)j * K + k) : make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    const int ti = blockIdx.x * NW + w;
    if (ti >= d_model / 16) return;
    const int i = lane & 15, gq = lane >> 4;
    const bf16_t* strip[1] = {wdown + ((size_t)ti * (Kp / 32) + k0 / 32) * tile<bf16_t>::kElems};
    f32x4_t acc[1] = {{0.f, 0.f, 0.f, 0.f}};
    mfma_strips<1, 8>(strip, len / 32, xs + (size_t)i * kpad + 8 * gq, i < M, acc);
    if (i < M) {
        float* dst = part + ((size_t)slice * M + i) * d_model + 16 * ti + 4 * gq;
        *reinterpret_cast<float4*>(dst) = make_float4(acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
    }
}

// ---------------------------------------------------------------------------------------------------------
bool skinny_supported(const cqil_dims& d, int P, int M) {
    (void)P;
    return d.dtype == CQIL_BF16 && M >= 2 && M <= 8 && d.d_model <= 8192;
}

template <typename K>
static hipError_t allow_lds(K kernel, size_t bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

hipError_t launch_skinny_step(const StepArgs& s, hipStream_t st) {
    const cqil_dims& d = s.d;
    const int P = s.P, dm = d.d_model, f = d.d_ffn, dk = d.head_dim, nh = d.n_heads;
    const int M = s.B * s.T;
    const bf16_t* wqkv = (const bf16_t*)(s.packed + s.pl.wqkv);
    const bf16_t* wo = (const bf16_t*)(s.packed + s.pl.wo);
    const bf16_t* wgu = (const bf16_t*)(s.packed + s.pl.wgu);
    const bf16_t* wdown = (const bf16_t*)(s.packed + s.pl.wdown);
    const bf16_t* g_attn = (const bf16_t*)(s.packed + s.pl.g_attn);
    const bf16_t* g_ffn = (const bf16_t*)(s.packed + s.pl.g_ffn);
    const float2* rope = (const float2*)(s.packed + s.pl.rope);
    float* q = (float*)(s.ws + s.wl.q);
    float* ctx = (float*)(s.ws + s.wl.ctx);
    float* a = (float*)(s.ws + s.wl.a);
    bf16_t* u = (bf16_t*)(s.ws + s.wl.u);
    float* dpart = (float*)(s.ws + s.wl.down_part);
    const int bd = s.bypass_d >= P ? P - 1 : s.bypass_d;
    const bf16_t* x = (const bf16_t*)s.x_in;
    hipError_t e;
#define CQIL_MARK(i) do { if (s.ev) (void)hipEventRecord(s.ev[i], st); } while (0)

    const size_t lds_full = (size_t)8 * (dm + kSkPad) * sizeof(bf16_t) + 64;
    CQIL_MARK(0);
    {
        constexpr int NW = 8;
        const int pairs = 3 * nh * (dk / 32);
        if ((e = allow_lds(qkv_skinny_kernel<NW>, lds_full)) != hipSuccess) return e;
        hipLaunchKernelGGL(HIP_KERNEL_NAME(qkv_skinny_kernel<NW>), dim3((pairs + NW - 1) / NW, P), dim3(NW * 64), lds_full,
                           st, x, wqkv, g_attn, rope, s.kv_len, (bf16_t*)s.kc, (bf16_t*)s.vc, q, M, s.T, dm, nh, dk,
                           d.max_seq, s.b_max, d.rms_eps);
    }
    CQIL_MARK(1);
    {
        const int lps = dk * 2 / 16;
#define CQIL_ATTN(LPS)                                                                                                \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(attn_decode_kernel<bf16_t, float, LPS, kAttnWaves>), dim3(P * M * nh),         \
                       dim3(kAttnThreads), 0, st, (const float*)q, (size_t)M * dm, (size_t)dm, (const bf16_t*)s.kc,        \
                       (const bf16_t*)s.vc, s.kv_len, ctx, M, s.T, nh, d.max_seq, s.b_max)
        switch (lps) {
            case 4: CQIL_ATTN(4); break;
            case 8: CQIL_ATTN(8); break;
            case 16: CQIL_ATTN(16); break;
            case 32: CQIL_ATTN(32); break;
            default: return hipErrorInvalidValue;
        }
#undef CQIL_ATTN
    }
    CQIL_MARK(2);
    {
        constexpr int NW = 4;
        if ((e = allow_lds(oproj_skinny_kernel<NW>, lds_full)) != hipSuccess) return e;
        hipLaunchKernelGGL(HIP_KERNEL_NAME(oproj_skinny_kernel<NW>), dim3((dm / 16 + NW - 1) / NW, P), dim3(NW * 64),
                           lds_full, st, ctx, wo, a, P, M, dm);
    }
    CQIL_MARK(3);
    {
        constexpr int NW = 8;
        if ((e = allow_lds(gateup_skinny_kernel<NW>, lds_full)) != hipSuccess) return e;
        hipLaunchKernelGGL(HIP_KERNEL_NAME(gateup_skinny_kernel<NW>), dim3((f / kGuBlock + NW - 1) / NW, P),
                           dim3(NW * 64), lds_full, st, x, a, wgu, g_ffn, u, P, bd, M, dm, f, d.rms_eps);
    }
    CQIL_MARK(4);
    {
        constexpr int NW = 8;
        const size_t lds = (size_t)8 * (s.wl.sk_slice + kSkPad) * sizeof(bf16_t);
        if ((e = allow_lds(down_skinny_kernel<NW>, lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(HIP_KERNEL_NAME(down_skinny_kernel<NW>), dim3((dm / 16 + NW - 1) / NW, s.wl.sk_slices),
                           dim3(NW * 64), lds, st, u, wdown, dpart, M, dm, P * f, s.wl.sk_slice);
    }
    CQIL_MARK(5);
    hipLaunchKernelGGL(HIP_KERNEL_NAME(merge_kernel<bf16_t>), dim3((dm + 255) / 256, M), dim3(256), 0, st, x, a, dpart,
                       (bf16_t*)s.x_out, s.kv_len, s.advance, P, s.wl.sk_slices, M, dm, s.B, s.T);
    CQIL_MARK(6);
#undef CQIL_MARK
    return hipGetLastError();
}

}  // namespace cqil
