// bf16 matrix-core GEMM of the token-parallel (prefill) path:  C[m][n] = sum_k A[m][k] * W[n][k]  (+ R[m][n]).
//
// A: activations, row-major [M][lda] bf16.  W: a packed weight matrix in the tiled layout (tile<> in cqil_dev.h),
// padded width Kp; a group z (blockIdx.z) addresses a row band (N-concatenation) or a column band
// (K-concatenation) of it.  C: row-major, bf16 or fp32; fp32 accumulation.
//
// Instruction: v_mfma_f32_32x32x16_bf16 (measured on gfx950: it sustains the full matrix rate in every arrangement
// with two waves per SIMD; the 16x16x32 form reaches 45 to 80 % of it, depending on the waves per SIMD and the
// independent accumulators it is given).  The weight rows are its A operand (lane i + 32 gg holds row i, columns 8 gg .. 8 gg + 7 of a
// 16-column slab), the tokens its B operand, so a lane ends up with groups of 4 consecutive weight rows of one
// token: 4 consecutive elements of a C row.
// A workgroup of WM x WN waves owns 32 TT WM tokens x 64 WN weight rows; a wave owns 32 TT tokens x 64 weight rows
// = TT x 2 instruction tiles (TT = 4: 128 accumulator registers; TT = 1 for up to 32 token rows).
// Weights never touch LDS: the packed layout stores every 16-row x 32-column tile in [column group][row] order,
// so the fragment of 32 rows x 16 columns is four contiguous 256-byte runs of two vertically adjacent tiles,
// which a wave reads straight from global memory, one 32-column slab ahead of use.
// Activations are staged in LDS as 1 KiB tiles of 32 tokens x 16 columns in operand order ([gg][token], 16-byte
// pieces), re-tiled on the way in; the piece of token j and piece index c of the 64-column step goes to slot
// (j + c) mod 32 of its half tile, so that the eight pieces of one 128-byte row segment, which eight neighbouring
// threads write, fall into different banks; every fragment read is one contiguous 16-byte-per-lane read.
// Two LDS stages of 64 columns: the global loads of step i+1 are in flight while step i is multiplied.
// All loads are unconditional with clamped addresses (no divergent branches in the loop): rows or strips outside
// the problem are computed from clamped data and never stored; columns beyond K are zeroed on the activation side.
#pragma once
#include "cqil_dev.h"

namespace cqil {

typedef __bf16 gemm_bf16x8 __attribute__((ext_vector_type(8)));
typedef float gemm_f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t gemm_u32x4 __attribute__((ext_vector_type(4)));

// buffer descriptors of the operand loads: raw buffers (stride 0) of 2 GiB from a wave-uniform base; the launcher
// checks that no offset reaches that range.  Word 3: 32-bit data format, no swizzle (the gfx9 / CDNA encoding).
constexpr uint32_t kGemmBufRange = 0x80000000u, kGemmBufFlags = 0x00020000u;

// epilogues: plain store, + fp32 residual R[m][n], SwiGLU over block-interleaved gate / up rows, or the rotary
// embedding of the QKV product with the KV-cache append
constexpr int kEpiNone = 0, kEpiAddR = 1, kEpiSwiglu = 2, kEpiRope = 3;

// Arguments of the kEpiRope epilogue (QKV product of one layer per group z, rows [q | k | v] of d_model each):
// q is rotated and stored to C, k is rotated and appended to the layer's K cache, v is appended to its V cache, at
// position kv_len[b] + t of token row m = b * T_new + t.  Requires d_model % 256 == 0 (a workgroup tile lies inside
// one of q, k, v) and head_dim 64 or 128 (a rotary pair meets in one lane, see RMAP).
struct GemmRope {
    const float2* rope;      // [max_seq][head_dim / 2] (cos, sin)
    const int32_t* kv_len;   // [b_max]
    bf16_t *kc, *vc;         // [groups][b_max][n_heads][max_seq][head_dim]
    int T_new, n_heads, d_k, max_seq, b_max, d_model;
};

__device__ __forceinline__ void gemm_store4(bf16_t* p, const float (&v)[4]) {
    uint2 o;
    o.x = f32x2_to_bf16x2(v[0], v[1]);
    o.y = f32x2_to_bf16x2(v[2], v[3]);
    *reinterpret_cast<uint2*>(p) = o;
}
__device__ __forceinline__ void gemm_store4(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}

// N, K: logical sizes of this group's product; N % 4 == 0, K % 8 == 0, M >= 1.  strip_step / ktile_step: group
// strides in 16-row strips / 32-column tiles inside W.  R (kEpiAddR): fp32 [M][N] added to the result.
// kEpiSwiglu: N % 32 == 0 rows as blocks of 16 gate + 16 up rows; C gets N / 2 columns per group.
// RMAP = 1 (head_dim 128 with kEpiRope): the wave's two 32-row fragments are rows e .. e + 31 and e + 64 .. e + 95
// of one head (e = 0 or 32), so that the rotary pair (e, e + 64) sits in the same lane and register of the two
// accumulator tiles; RMAP = 0: rows 64 wn .. 64 wn + 63 (for head_dim 64 that already pairs e with e + 32).
template <typename CT, int EPI, int WM, int WN, int TT, bool WSTREAM, int RMAP = 0>
__global__ __launch_bounds__(64 * WM * WN, 2) void gemm_mfma_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, CT* __restrict__ C, const float* __restrict__ R, int M,
    int N, int K, size_t lda, size_t Kp, size_t ldc, int groups, size_t sA, size_t strip_step, size_t ktile_step,
    size_t sC, int ksplit, float* __restrict__ part, GemmRope rp) {
    constexpr int BM = 32 * TT * WM, BN = 64 * WN, NT = 64 * WM * WN;
    constexpr int TE = 512;            // elements per tile
    constexpr int STAGE = BM * 64;     // activation elements per LDS stage
    constexpr int APT = BM * 8 / NT;   // activation pieces per thread and step
    extern __shared__ __align__(16) unsigned char gemm_smem[];
    bf16_t* lds = reinterpret_cast<bf16_t*>(gemm_smem);
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int wm = w / WN, wn = w % WN;
    // Workgroup -> tile.  The hardware deals consecutive workgroups of the 1-D grid to the 8 XCDs in turn, and
    // each XCD has its own L2: the workgroups that run together on one XCD (every 8th) are given a compact
    // block of SM x SN tiles, so that they share SM activation bands and SN weight bands in that L2.
    constexpr int SN = 8, SM = (WM * WN == 8) ? 4 : 8, ST = SM * SN;
    const int nx = (N + BN - 1) / BN, ny = (M + BM - 1) / BM;
    const int snx = (nx + SN - 1) / SN, sny = (ny + SM - 1) / SM;
    const int L = blockIdx.x, idx = L >> 3;
    const int S = (idx / ST) * 8 + (L & 7), t = idx % ST;
    const int zk = S / (snx * sny), s2 = S % (snx * sny);
    const int z = zk / ksplit, ks = zk % ksplit;  // group, K slice (split-K: partial sums go to `part`)
    // Super-tiles are walked down the token axis first: the 8 XCDs, which take consecutive super-tiles, then work
    // on the same band of weight rows at the same time (one fetch from HBM, shared through the last-level cache)
    // and the activations (which fit that cache whole) are what each XCD re-reads per band.  Walking along the
    // weight rows first streamed every weight band from HBM once per token band: 3-4 % slower on the wide products.
    const int nt = (s2 / sny) * SN + t % SN, mt = (s2 % sny) * SM + t / SN;
    if (z >= groups || nt >= nx || mt >= ny) return;  // padding of the grid (uniform for the workgroup)
    A += (size_t)z * sA;
    C += (size_t)z * sC;
    const int m0 = mt * BM, n0 = nt * BN;
    const size_t w_tiles_per_strip = Kp / 32;
    const int n_strips = (N + 15) / 16;
    const int n_ktiles = (K + 31) / 32;
    const int n_steps = (n_ktiles + 1) / 2;

    // weight fragments: rows 32 s .. 32 s + 31 of the wave's 64 = strips 4 wn + 2 s + (i >> 4); lane (i, gg) reads
    // piece (2 hf + gg) * 16 + (i & 15) of tile kt for the 16-column slab k16 = 2 kt + hf: 256 elements per slab
    const int fi = lane & 31, fgg = lane >> 5;
    const int n_k16 = 2 * n_ktiles;
    // Both operands come by buffer loads (wave-uniform base in scalar registers + a per-lane byte offset fixed for
    // the whole product + a wave-uniform offset per slab / step): no per-lane address arithmetic in the loop.
    const bf16_t* wbase = W + (((size_t)z * strip_step + n0 / 16) * w_tiles_per_strip + (size_t)z * ktile_step) * TE;
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(wbase), 0, kGemmBufRange, kGemmBufFlags);
    uint32_t wvo[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int row_base = RMAP ? 128 * (wn >> 1) + 32 * (wn & 1) + 64 * s : 64 * wn + 32 * s;  // of the tile's 256
        const int rel = min(row_base / 16 + (fi >> 4), n_strips - 1 - n0 / 16);
        wvo[s] = (uint32_t)(((size_t)rel * w_tiles_per_strip * TE + (fgg * 16 + (fi & 15)) * 8) * 2);
    }
    // WSTREAM: a single band of token tiles reads every weight once: streaming (non-temporal) loads
    constexpr int kWeightAux = WSTREAM ? 2 : 0;
    gemm_u32x4 wf[4][2];  // [slab of the step][s]
    auto load_w = [&](int b, int k16) {
        const uint32_t soff = (uint32_t)min(k16, n_k16 - 1) * 512u;
#pragma unroll
        for (int s = 0; s < 2; ++s) wf[b][s] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wvo[s], soff, kWeightAux);
    };

    // activation pieces: thread -> (row, 16-byte piece c) of the 64-column step, APT rows NT/8 apart
    const int c = tid & 7;
    const __amdgpu_buffer_rsrc_t arsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(A + (size_t)m0 * lda), 0, kGemmBufRange, kGemmBufFlags);
    uint32_t avo[APT];
    int a_lds[APT];
#pragma unroll
    for (int q = 0; q < APT; ++q) {
        const int row = (tid >> 3) + (NT / 8) * q;
        avo[q] = (uint32_t)(((size_t)min(row, M - 1 - m0) * lda + 8 * c) * 2);
        const int ts = row >> 5, j = row & 31, k16 = c >> 1, gg = c & 1;
        a_lds[q] = (ts * 4 + k16) * TE + (gg * 32 + ((j + c) & 31)) * 8;
    }
    // In the last step a piece may lie past column K: it is read from columns K - 8 .. K - 1 instead (a_tail < 0
    // moves the lane there) and replaced by zeros when it goes to LDS.  Steps past the last read the last again.
    const int last_step = n_steps - 1;
    const int a_tail = (64 * last_step + 8 * c < K) ? 0 : 2 * (K - 8 - 64 * last_step - 8 * c);
    gemm_u32x4 areg[APT];
    uint32_t a_keep = 0;  // all ones if the loaded columns exist, else zero (applied when the pieces go to LDS)
    auto load_a = [&](int step) {
        a_keep = (64 * step + 8 * c < K) ? 0xffffffffu : 0u;
        const uint32_t soff = (uint32_t)min(step, last_step) * 128u;
        const int adj = step >= last_step ? a_tail : 0;
#pragma unroll
        for (int q = 0; q < APT; ++q)
            areg[q] = __builtin_amdgcn_raw_buffer_load_b128(arsrc, avo[q] + (uint32_t)adj, soff, 0);
    };
    auto store_a = [&](bf16_t* as) {
#pragma unroll
        for (int q = 0; q < APT; ++q)
            *reinterpret_cast<uint4*>(as + a_lds[q]) =
                make_uint4(areg[q][0] & a_keep, areg[q][1] & a_keep, areg[q][2] & a_keep, areg[q][3] & a_keep);
    };

    gemm_f32x16 acc[TT][2];
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][s][r] = 0.f;

    // activation fragment of token tile t, slab k16 of the step: tile (4 wm + t) * 4 + k16, slot (j + 2 k16 + gg) mod 32
    int frag[4];
#pragma unroll
    for (int k16 = 0; k16 < 4; ++k16) frag[k16] = (TT * wm * 4 + k16) * TE + (fgg * 32 + ((fi + 2 * k16 + fgg) & 31)) * 8;
    auto read_af = [&](uint4(&af)[TT], const bf16_t* as, int k16) {
#pragma unroll
        for (int t = 0; t < TT; ++t) af[t] = *reinterpret_cast<const uint4*>(as + frag[k16] + t * 4 * TE);
    };
    auto mma = [&](const uint4(&af)[TT], int b) {
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int s = 0; s < 2; ++s)
                acc[t][s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(gemm_bf16x8, wf[b][s]),
                                                                    __builtin_bit_cast(gemm_bf16x8, af[t]), acc[t][s], 0, 0, 0);
    };

    // Software pipeline, one slab (16 columns, 2 TT instructions) per stage: the fragments of slab b+1 are read
    // from LDS while the instructions of slab b issue, the weights of a slab are fetched a whole step ahead, the
    // activations two steps ahead, and the next step's activations are written to the other LDS stage during the
    // third slab, so that the single barrier of a step is passed while those are in the pipe.  Within a stage the
    // scheduling groups spread the memory instructions one by one between the matrix instructions (issued in a
    // burst they cost about 8 % of the throughput); the scheduling barriers keep the stages apart.
    uint4 afa[TT], afb[TT];
    const int steps_per_slice = (n_steps + ksplit - 1) / ksplit;
    const int s_beg = ks * steps_per_slice, s_end = min(s_beg + steps_per_slice, n_steps);  // may be empty
    load_a(s_beg);
#pragma unroll
    for (int b = 0; b < 4; ++b) load_w(b, 4 * s_beg + b);
    store_a(lds);
    load_a(s_beg + 1);
    __syncthreads();
    read_af(afa, lds, 0);
    constexpr int kMfma = 0x008, kVmemRd = 0x020, kDsRd = 0x100, kDsWr = 0x200;  // scheduling group masks
    for (int step = s_beg; step < s_end; ++step) {
        bf16_t* cur = lds + ((step - s_beg) & 1) * STAGE;
        bf16_t* nxt = lds + (((step - s_beg) & 1) ^ 1) * STAGE;
        const int k16n = 4 * (step + 1);
        read_af(afb, cur, 1);
        mma(afa, 0);
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            __builtin_amdgcn_sched_group_barrier(kDsRd, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kMfma, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_w(0, k16n);
        read_af(afa, cur, 2);
        mma(afb, 1);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            __builtin_amdgcn_sched_group_barrier(kVmemRd, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        }
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            __builtin_amdgcn_sched_group_barrier(kDsRd, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_w(1, k16n + 1);
        read_af(afb, cur, 3);
        store_a(nxt);  // beyond the last step: zeros, stored to the idle stage and never used
        load_a(step + 2);
        mma(afa, 2);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            __builtin_amdgcn_sched_group_barrier(kVmemRd, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        }
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            __builtin_amdgcn_sched_group_barrier(kDsRd, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        }
#pragma unroll
        for (int q = 0; q < APT; ++q) {
            __builtin_amdgcn_sched_group_barrier(kDsWr, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kVmemRd, 1, 0);
            if (q < TT - 2) __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_w(2, k16n + 2);
        __syncthreads();
        read_af(afa, nxt, 0);
        mma(afb, 3);
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            __builtin_amdgcn_sched_group_barrier(kDsRd, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kMfma, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_w(3, k16n + 3);
    }

    // ---- epilogue: lane (j, h) holds, in registers 4 q .. 4 q + 3, weight rows 8 q + 4 h .. + 3 of token j
    if (ksplit > 1) {  // partial sums of this K slice: part[ks][z][m][n], fp32; gemm_reduce_kernel finishes
        float* pz = part + ((size_t)ks * groups + z) * (size_t)M * N;
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const int m = m0 + 32 * TT * wm + 32 * t + fi;
            if (m >= M) continue;
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + 64 * wn + 32 * s + 8 * q + 4 * fgg;
                    if (n >= N) continue;
                    *reinterpret_cast<float4*>(pz + (size_t)m * N + n) =
                        make_float4(acc[t][s][4 * q], acc[t][s][4 * q + 1], acc[t][s][4 * q + 2], acc[t][s][4 * q + 3]);
                }
        }
        return;
    }
    if constexpr (EPI == kEpiRope) {
        // fragment 0 holds rows e .. e + 31 of the first half of a head, fragment 1 the partner rows e + d_k / 2
        const int half = rp.d_k >> 1;
        const int nb0 = n0 + (RMAP ? 128 * (wn >> 1) + 32 * (wn & 1) : 64 * wn);  // first row of fragment 0
        if (nb0 >= N) return;
        const int sec = nb0 / rp.d_model, nn = nb0 % rp.d_model;  // 0 = q, 1 = k, 2 = v (uniform for the wave)
        const int h = nn / rp.d_k, e0 = nn % rp.d_k;
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const int m = m0 + 32 * TT * wm + 32 * t + fi;
            if (m >= M) continue;
            const int b = m / rp.T_new, pos = rp.kv_len[b] + m % rp.T_new;
            const bool pos_ok = pos >= 0 && pos < rp.max_seq;
            bf16_t* dst;
            if (sec == 0) {
                dst = reinterpret_cast<bf16_t*>(C) + (size_t)m * ldc + nb0;
            } else {
                if (!pos_ok) continue;
                dst = (sec == 1 ? rp.kc : rp.vc) +
                      ((((size_t)z * rp.b_max + b) * rp.n_heads + h) * (size_t)rp.max_seq + pos) * rp.d_k + e0;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = 8 * q + 4 * fgg;   // offset inside the fragment: pair index e0 + e .. + 3
                float lo[4], hi[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) { lo[i] = acc[t][0][4 * q + i]; hi[i] = acc[t][1][4 * q + i]; }
                if (sec < 2 && pos_ok) {
                    const float4* cs = reinterpret_cast<const float4*>(rp.rope + (size_t)pos * half + e0 + e);
                    const float4 c01 = cs[0], c23 = cs[1];
                    const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float a = lo[i], bb = hi[i];
                        lo[i] = a * co[i] - bb * si[i];
                        hi[i] = bb * co[i] + a * si[i];
                    }
                }
                gemm_store4(dst + e, lo);
                gemm_store4(dst + e + half, hi);
            }
        }
        return;
    }
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        const int m = m0 + 32 * TT * wm + 32 * t + fi;
        if (m >= M) continue;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (EPI == kEpiSwiglu) {
                // rows come as 16 gate rows followed by their 16 up rows: gate row 8 q + 4 h + e (q = 0, 1) and
                // its up row sit in the same lane, registers 4 q + e and 4 (q + 2) + e.  Output column of the
                // group: 16 (row block) + 8 q + 4 h + e; N counts gate and up rows, ldc / sC are those of u.
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int n = n0 + 64 * wn + 32 * s + 8 * q + 4 * fgg;   // gate row
                    if (n >= N) continue;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float gte = acc[t][s][4 * q + e], up = acc[t][s][4 * (q + 2) + e];
                        v[e] = gte / (1.0f + __expf(-gte)) * up;
                    }
                    gemm_store4(C + (size_t)m * ldc + (n0 + 64 * wn + 32 * s) / 2 + 8 * q + 4 * fgg, v);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + 64 * wn + 32 * s + 8 * q + 4 * fgg;
                    if (n >= N) continue;
                    float v[4] = {acc[t][s][4 * q], acc[t][s][4 * q + 1], acc[t][s][4 * q + 2], acc[t][s][4 * q + 3]};
                    if (EPI == kEpiAddR) {
                        const float4 r = *reinterpret_cast<const float4*>(R + (size_t)m * N + n);
                        v[0] += r.x; v[1] += r.y; v[2] += r.z; v[3] += r.w;
                    }
                    gemm_store4(C + (size_t)m * ldc + n, v);
                }
            }
        }
    }
}

// C[z][m][n] = sum_ks part[ks][z][m][n] (+ R[m][n]), 4 elements per thread
template <typename CT, int EPI>
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float* __restrict__ part, CT* __restrict__ C,
                                                          const float* __restrict__ R, int M, int N, size_t ldc,
                                                          int groups, size_t sC, int ksplit) {
    const size_t per_group = (size_t)M * N / 4, total = per_group * groups;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t z = i / per_group, e = (i % per_group) * 4;
        const size_t m = e / N, n = e % N;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        for (int ks = 0; ks < ksplit; ++ks) {
            const float4 p4 = *reinterpret_cast<const float4*>(part + (((size_t)ks * groups + z) * M + m) * N + n);
            v[0] += p4.x; v[1] += p4.y; v[2] += p4.z; v[3] += p4.w;
        }
        if (EPI == kEpiAddR) {
            const float4 r = *reinterpret_cast<const float4*>(R + m * N + n);
            v[0] += r.x; v[1] += r.y; v[2] += r.z; v[3] += r.w;
        }
        gemm_store4(C + z * sC + m * ldc + n, v);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Up to 32 token rows (a batch of decode rows): the product is a weight stream.  A workgroup of 4 waves owns 64
// weight rows; the waves split its K range four ways and never meet before the end: every wave fetches its own
// weight fragments and its own activation fragments (32 rows x 16 columns straight from global memory, they stay
// in L2) a ring of kRowsRing slabs ahead, no LDS staging, no barrier in the loop.  The four partial tiles are
// added through LDS in wave order; wave w then finishes rows 8 (w & 1) + {0..7 of 16, and the 8 rows 16 further}
// of row block w >> 1 (for SwiGLU that is a gate quad and its up quad).  Many small workgroups (ten or more
// waves per SIMD pair fit) keep far more bytes in flight per CU than the tiled kernel's two workgroups.
// ---------------------------------------------------------------------------------------------------------
constexpr int kRowsRing = 4;
template <typename CT, int EPI>
__global__ __launch_bounds__(256) void gemm_rows_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, CT* __restrict__ C, const float* __restrict__ R, int M,
    int N, int K, size_t lda, size_t Kp, size_t ldc, int groups, size_t sA, size_t strip_step, size_t ktile_step,
    size_t sC, int ksplit, float* __restrict__ part) {
    constexpr int TE = 512;
    __shared__ __align__(16) float red[4][32][64];   // [wave][accumulator register][lane]
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int fi = lane & 31, fgg = lane >> 5;
    const int nx = (N + 63) / 64;
    const int nt = blockIdx.x % nx, zk = blockIdx.x / nx;
    const int z = zk / ksplit, ks = zk % ksplit;
    if (z >= groups) return;
    A += (size_t)z * sA;
    C += (size_t)z * sC;
    const int n0 = nt * 64;
    const size_t w_tiles_per_strip = Kp / 32;
    const int n_strips = (N + 15) / 16;
    const int n_k16 = 2 * (int)((K + 31) / 32);
    // slabs of this workgroup's K slice, then of this wave's quarter of it
    const int per_slice = (n_k16 + ksplit - 1) / ksplit;
    const int g0 = min(ks * per_slice, n_k16), g1 = min(g0 + per_slice, n_k16);
    const int per_wave = (g1 - g0 + 3) / 4;
    const int k0 = min(g0 + w * per_wave, g1), k1 = min(k0 + per_wave, g1);

    const bf16_t* wbase = W + (((size_t)z * strip_step + n0 / 16) * w_tiles_per_strip + (size_t)z * ktile_step) * TE;
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(wbase), 0, kGemmBufRange, kGemmBufFlags);
    const __amdgpu_buffer_rsrc_t arsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(A), 0, kGemmBufRange, kGemmBufFlags);
    uint32_t wvo[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int rel = min(2 * s + (fi >> 4), n_strips - 1 - n0 / 16);
        wvo[s] = (uint32_t)(((size_t)rel * w_tiles_per_strip * TE + (fgg * 16 + (fi & 15)) * 8) * 2);
    }
    const uint32_t avo = (uint32_t)(((size_t)min(fi, M - 1) * lda + 8 * fgg) * 2);

    gemm_u32x4 wf[kRowsRing][2], af[kRowsRing];
    auto request = [&](int slot, int k16) {
        const int kc = min(k16, n_k16 - 1);
        // activation columns past K (inside the last 32-column tile) are read from the last piece of the row
        // and dropped below; the weights there are the packer's zero padding
        const int col = min(16 * kc + 8 * fgg, K - 8);
        af[slot] = __builtin_amdgcn_raw_buffer_load_b128(arsrc, avo + (uint32_t)(2 * (col - 8 * fgg)), 0, 0);
#pragma unroll
        for (int s = 0; s < 2; ++s)
            wf[slot][s] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wvo[s], (uint32_t)kc * 512u, 2);  // streamed once
    };
    gemm_f32x16 acc[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[s][r] = 0.f;
#pragma unroll
    for (int i = 0; i < kRowsRing; ++i) request(i, k0 + i);
    for (int kb = k0; kb < k1; kb += kRowsRing) {
#pragma unroll
        for (int i = 0; i < kRowsRing; ++i) {
            if (kb + i < k1) {  // wave-uniform
                gemm_u32x4 a = af[i];
                if (16 * (kb + i) + 8 * fgg >= K) a = gemm_u32x4{0u, 0u, 0u, 0u};
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(gemm_bf16x8, wf[i][s]),
                                                                     __builtin_bit_cast(gemm_bf16x8, a), acc[s], 0, 0, 0);
                if (kb + i + kRowsRing < k1) request(i, kb + i + kRowsRing);
            }
        }
    }
    // ---- the four K quarters meet: partial tiles through LDS, added in wave order
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[w][16 * s + r][lane] = acc[s][r];
    __syncthreads();
    const int s_out = w >> 1, qp = w & 1;   // this wave finishes registers 4 qp .. + 3 and 4 (qp + 2) .. + 3 of block s_out
    float v[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int reg = 16 * s_out + 4 * (qp + 2 * half) + e;
            v[half][e] = ((red[0][reg][lane] + red[1][reg][lane]) + red[2][reg][lane]) + red[3][reg][lane];
        }
    const int m = fi;
    if (m >= M) return;
    const int nb = n0 + 32 * s_out;  // first weight row of the block
    if (ksplit > 1) {  // partial sums of this K slice: part[ks][z][m][n], fp32; gemm_reduce_kernel finishes
        float* pz = part + ((size_t)ks * groups + z) * (size_t)M * N;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int n = nb + 8 * (qp + 2 * half) + 4 * fgg;
            if (n < N) *reinterpret_cast<float4*>(pz + (size_t)m * N + n) = make_float4(v[half][0], v[half][1], v[half][2], v[half][3]);
        }
        return;
    }
    if (EPI == kEpiSwiglu) {
        const int n = nb + 8 * qp + 4 * fgg;  // gate row; its up row is 16 further
        if (n < N) {
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = v[0][e] / (1.0f + __expf(-v[0][e])) * v[1][e];
            gemm_store4(C + (size_t)m * ldc + nb / 2 + 8 * qp + 4 * fgg, o);
        }
    } else {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int n = nb + 8 * (qp + 2 * half) + 4 * fgg;
            if (n >= N) continue;
            float o[4] = {v[half][0], v[half][1], v[half][2], v[half][3]};
            if (EPI == kEpiAddR) {
                const float4 r = *reinterpret_cast<const float4*>(R + (size_t)m * N + n);
                o[0] += r.x; o[1] += r.y; o[2] += r.z; o[3] += r.w;
            }
            gemm_store4(C + (size_t)m * ldc + n, o);
        }
    }
}

template <typename CT, int EPI>
static hipError_t gemm_rows_launch(const bf16_t* A, const bf16_t* W, CT* C, const float* R, int M, int N, int K,
                                   size_t lda, size_t Kp, size_t ldc, int groups, size_t sA, size_t n_step,
                                   size_t k_step, size_t sC, float* part, size_t part_floats, hipStream_t st) {
    const int nx = (N + 63) / 64;
    const long tiles = (long)nx * groups;
    const int n_k16 = 2 * ((K + 31) / 32);
    // K slices across workgroups until about a thousand workgroups (15 waves per CU) exist; a wave keeps 8 slabs or
    // more.  (13B, 8 rows: O projection 35 us with 1280 workgroups, 41 us with 640.)
    int ksplit = 1;
    if (EPI != kEpiSwiglu && part != nullptr) {
        const size_t per_slice = (size_t)groups * M * N;
        while (ksplit < 16 && tiles * ksplit < 960 && n_k16 / (ksplit * 2 * 4) >= 8 &&
               per_slice * (size_t)(ksplit * 2) <= part_floats)
            ksplit *= 2;
    }
    const long wgs = tiles * ksplit;
    if (wgs > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_rows_kernel<CT, EPI>), dim3((unsigned)wgs), dim3(256), 0, st, A, W, C, R, M, N, K,
                       lda, Kp, ldc, groups, sA, n_step / 16, k_step / 32, sC, ksplit, part);
    if (ksplit > 1) {
        const size_t total = (size_t)groups * M * N / 4;
        const unsigned g = (unsigned)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
        hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_reduce_kernel<CT, EPI>), dim3(g), dim3(256), 0, st, part, C, R, M, N, ldc,
                           groups, sC, ksplit);
    }
    return hipSuccess;
}

// Same argument convention as the plain kernel of the token-parallel path: n_step / k_step are the group strides
// in weight rows / columns (multiples of 16 / 32).  part / part_floats: scratch for split-K partial sums (may be
// null / 0): when the tile grid is too small to fill the chip, K is cut into slices of whole 64-column steps,
// each slice writes fp32 partial sums and a second kernel adds them in slice order (deterministic).
template <typename CT, int EPI, int WM, int WN, int TT>
static hipError_t gemm_mfma_launch(const bf16_t* A, const bf16_t* W, CT* C, const float* R, int M, int N, int K,
                                   size_t lda, size_t Kp, size_t ldc, int groups, size_t sA, size_t n_step,
                                   size_t k_step, size_t sC, float* part, size_t part_floats, hipStream_t st) {
    constexpr int BM = 32 * TT * WM, BN = 64 * WN;
    // TT == 1 needs 8 KiB but asks for 64: that keeps two workgroups per CU.  With more resident per CU the
    // dispatcher packs a grid of a few hundred workgroups onto a part of the chip (measured: CUs busy 60 % of the
    // kernel, 260 us against 187 us for the 13B gate/up product with 8 rows).
    constexpr size_t lds_bytes = TT == 1 ? 65536 : 2 * (size_t)BM * 64 * 2;
    constexpr int SN = 8, SM = (WM * WN == 8) ? 4 : 8;
    const int nx = (N + BN - 1) / BN, ny = (M + BM - 1) / BM;
    int ksplit = 1;
    if (EPI != kEpiSwiglu && part != nullptr) {
        const long tiles = (long)nx * ny * groups;
        const int n_steps = (K + 63) / 64;
        const size_t per_slice = (size_t)groups * M * N;
        while (ksplit < 16 && tiles * ksplit < 384 && n_steps / (ksplit * 2) >= 8 &&
               per_slice * (size_t)(ksplit * 2) <= part_floats)
            ksplit *= 2;
    }
    const long supers = (long)groups * ksplit * ((nx + SN - 1) / SN) * ((ny + SM - 1) / SM);
    const long wgs = (supers + 7) / 8 * 8 * SM * SN;
    if (wgs > 0x7fffffffL) return hipErrorInvalidValue;
    if (ny == 1)
        hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_mfma_kernel<CT, EPI, WM, WN, TT, true>), dim3((unsigned)wgs),
                           dim3(64 * WM * WN), lds_bytes, st, A, W, C, R, M, N, K, lda, Kp, ldc, groups, sA, n_step / 16,
                           k_step / 32, sC, ksplit, part, GemmRope{});
    else
        hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_mfma_kernel<CT, EPI, WM, WN, TT, false>), dim3((unsigned)wgs),
                           dim3(64 * WM * WN), lds_bytes, st, A, W, C, R, M, N, K, lda, Kp, ldc, groups, sA, n_step / 16,
                           k_step / 32, sC, ksplit, part, GemmRope{});
    if (ksplit > 1) {
        const size_t total = (size_t)groups * M * N / 4;
        const unsigned g = (unsigned)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
        hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_reduce_kernel<CT, EPI>), dim3(g), dim3(256), 0, st, part, C, R, M, N, ldc,
                           groups, sC, ksplit);
    }
    return hipSuccess;
}

// QKV product with the rotary embedding and the KV append in the epilogue (see GemmRope): M > 32 token rows, no
// split along K, 128 x 256 tiles.  A [groups][M][K] (sA apart), W rows [q | k | v] of each group n_step apart.
static hipError_t gemm_mfma_qkv_rope(const bf16_t* A, const bf16_t* W, bf16_t* C, int M, int N, int K, size_t lda, size_t Kp,
                                     size_t ldc, int groups, size_t sA, size_t n_step, size_t sC, const GemmRope& rp,
                                     hipStream_t st) {
    if (M <= 32 || (N & 255) || (K & 7) || K < 8 || rp.d_model % 256 || N != 3 * rp.d_model ||
        (rp.d_k != 64 && rp.d_k != 128))
        return hipErrorInvalidValue;
    if (Kp >= (1u << 21) || lda >= (1u << 21)) return hipErrorInvalidValue;
    constexpr int BM = 128, BN = 256, SN = 8, SM = 8;
    const int nx = (N + BN - 1) / BN, ny = (M + BM - 1) / BM;
    const long supers = (long)groups * ((nx + SN - 1) / SN) * ((ny + SM - 1) / SM);
    const long wgs = (supers + 7) / 8 * 8 * SM * SN;
    if (wgs > 0x7fffffffL) return hipErrorInvalidValue;
    constexpr size_t lds_bytes = 2 * (size_t)BM * 64 * 2;
    if (rp.d_k == 128)
        hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_mfma_kernel<bf16_t, kEpiRope, 1, 4, 4, false, 1>), dim3((unsigned)wgs), dim3(256),
                           lds_bytes, st, A, W, C, nullptr, M, N, K, lda, Kp, ldc, groups, sA, n_step / 16, 0, sC, 1, nullptr, rp);
    else
        hipLaunchKernelGGL(HIP_KERNEL_NAME(gemm_mfma_kernel<bf16_t, kEpiRope, 1, 4, 4, false, 0>), dim3((unsigned)wgs), dim3(256),
                           lds_bytes, st, A, W, C, nullptr, M, N, K, lda, Kp, ldc, groups, sA, n_step / 16, 0, sC, 1, nullptr, rp);
    return hipSuccess;
}

// tile: 1 = 256 tokens x 256 rows (8 waves), 2 = 128 x 256 (4 waves) also for few rows; 0 = default
template <typename CT, int EPI>
static hipError_t gemm_mfma(int tile_sel, const bf16_t* A, const bf16_t* W, CT* C, const float* R, int M, int N, int K,
                            size_t lda, size_t Kp, size_t ldc, int groups, size_t sA, size_t n_step, size_t k_step,
                            size_t sC, hipStream_t st, float* part = nullptr, size_t part_floats = 0) {
    if (M < 1 || (N & 3) || (K & 7) || K < 8) return hipErrorInvalidValue;
    if (Kp >= (1u << 21) || lda >= (1u << 21)) return hipErrorInvalidValue;  // byte offsets of a tile stay below 2 GiB
    // default: 128 x 256 (two workgroups per CU overlap each other's barriers and load latency)
    // up to 8 token rows, plain and residual epilogues (QKV, O, down): the barrier-free streaming kernel.  Measured at
    // the 13B shape, P = 4, against the tiled kernel with one 32-token tile per wave: O projection 34 against 41 us,
    // down 85 against 95, QKV 99 against 98 + 5 for the K-slice reduction it needs; from 16 rows on the per-wave
    // activation fragments cost more than the barriers saved (QKV 125 against 102 us), and the gate/up product is
    // faster tiled at every row count (166 against 170 us).  tile_sel 2 forces the tiled kernel.
    if (M <= 8 && EPI != kEpiSwiglu && tile_sel != 2)
        return gemm_rows_launch<CT, EPI>(A, W, C, R, M, N, K, lda, Kp, ldc, groups, sA, n_step, k_step, sC, part,
                                         part_floats, st);
    if (M <= 32)
        return gemm_mfma_launch<CT, EPI, 1, 4, 1>(A, W, C, R, M, N, K, lda, Kp, ldc, groups, sA, n_step, k_step, sC, part,
                                                  part_floats, st);
    if (tile_sel == 1)
        return gemm_mfma_launch<CT, EPI, 2, 4, 4>(A, W, C, R, M, N, K, lda, Kp, ldc, groups, sA, n_step, k_step, sC, part,
                                               part_floats, st);
    return gemm_mfma_launch<CT, EPI, 1, 4, 4>(A, W, C, R, M, N, K, lda, Kp, ldc, groups, sA, n_step, k_step, sC, part,
                                           part_floats, st);
}

}  // namespace cqil
