// Causal attention of the token-parallel (prefill) path on the matrix cores, bf16:
//   softmax(Q K^T / sqrt(d_k)) V  (Eq.2)  for the T new tokens of every (layer, sequence, head), over the cached
//   slots and the new tokens up to and including the query (positions kv_len[b] + t).
//
// Transposed formulation, so that nothing has to be re-laid out between the two products:
//   S^T[key][query] = K Q^T     A operand = K rows (i = key), B operand = Q rows (j = query)
//   O^T[d][query]   = V^T P^T   A operand = V^T (i = d),      B operand = P^T  (j = query)
// With v_mfma_f32_16x16x32_bf16 the result lane j + 16 g holds rows 4g..4g+3 of column j: after the first product
// a lane owns four consecutive keys of one query in each 16-key tile; two such tiles give it eight keys, which is
// exactly one B-operand fragment of the second product if the instruction's k slots (g, e) are taken to mean key
// 16 a + 4 g + e for e < 4 and 16 b + 4 g + e - 4 for e >= 4 (a, b the two tiles).  V^T is staged in LDS in that
// same key order, so P stays in registers.  The softmax statistics of a query live in the four lanes that share
// its column (two cross-lane steps), the running maximum / sum / output are rescaled per key tile (online softmax).
//
// Workgroup: 4 waves, 128 queries (32 per wave: two column tiles), key tiles of 64.  K tile and V^T tile are
// staged in LDS as 1 KiB tiles in A-operand order, in two stages: while a tile is multiplied the next one goes
// from registers to the other stage and the one after that is fetched (one barrier per tile).  V is transposed in registers: a thread fetches 4 values of d for the 8 keys of
// one operand piece and writes 4 complete 16-byte pieces (no sub-word LDS writes).
#pragma once
#include "cqil_dev.h"

namespace cqil {

typedef __bf16 attn_bf16x8 __attribute__((ext_vector_type(8)));
typedef float attn_f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPfBQ = 128, kPfBKV = 64, kPfThreads = 256;
constexpr int kPfUnitGroup = 8;  // head units whose query blocks are interleaved on one XCD

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    return f32x2_to_bf16x2(a, b);
}

template <int DK>
__global__ __launch_bounds__(kPfThreads, 2) void attn_prefill_mfma_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc,
    const int32_t* __restrict__ kv_len, bf16_t* __restrict__ ctx, int P, int B, int T_new, int n_heads, int max_seq,
    int b_max) {
    constexpr int NDB = DK / 32;  // 32-wide d blocks (k steps of the first product)
    constexpr int NDT = DK / 16;  // 16-row d tiles (row tiles of the second product)
    constexpr int PPK = DK / 8;   // 16-byte pieces per key row
    constexpr int TE = 512;
    constexpr int KPT = (kPfBKV * PPK) / kPfThreads;        // K pieces per thread and tile
    constexpr int NVG = (kPfBKV / 8) * (DK / 4);            // V groups (8 keys x 4 d) of a tile
    constexpr int VG = (NVG + kPfThreads - 1) / kPfThreads;  // per thread (the last round may be partial: whole waves)
    static_assert(KPT >= 1 && NVG % 64 == 0, "tile too small for the workgroup");
    constexpr int KSZ = 4 * NDB * TE, VSZ = NDT * 2 * TE;
    __shared__ __align__(16) bf16_t Ks2[2 * KSZ];   // two stages of [key tile 0..3][d block]
    __shared__ __align__(16) bf16_t Vs2[2 * VSZ];   // two stages of [d tile][key block 0..1]

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int j = lane & 15, g = lane >> 4;
    // Workgroup -> (head unit, query block).  The hardware deals consecutive workgroups of the 1-D grid to the 8
    // XCDs in turn, and each XCD has its own L2: unit u = (layer, sequence, head) is given to XCD u mod 8, so its keys
    // and values are fetched into one L2 only and all its query blocks find them there.  On an XCD, units are taken
    // kPfUnitGroup at a time and their query blocks longest (latest) first: the 64 workgroups an XCD runs at once
    // are then a mix of long and short blocks of a few units.  (With a 2-D grid of query block x unit every XCD read
    // every unit: 1.12 ms against 0.70 ms at 13B, P=2, B=4, T=2048.)
    const int nqb = (T_new + kPfBQ - 1) / kPfBQ, units = P * B * n_heads;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int grp = slot / (kPfUnitGroup * nqb), i_in = slot % (kPfUnitGroup * nqb);
    const int qb = nqb - 1 - i_in / kPfUnitGroup;
    const int unit = xcd + 8 * (grp * kPfUnitGroup + i_in % kPfUnitGroup);
    if (unit >= units) return;  // padding of the grid (whole workgroup)
    const int h = unit % n_heads;
    const int lb = unit / n_heads;
    const int b = lb % B, l = lb / B;
    const int M = B * T_new;
    const size_t d_model = (size_t)n_heads * DK;
    const int S_b = kv_len[b];
    const int q0 = qb * kPfBQ + 32 * w;
    // keys this workgroup needs: the cache plus the new tokens up to its last query
    int kv_end = S_b + min(qb * kPfBQ + kPfBQ, T_new);
    if (kv_end > max_seq) kv_end = max_seq;
    if (kv_end < 1) return;  // a negative kv_len: nothing to read (whole workgroup)
    const size_t head_off = ((((size_t)l * b_max + b) * n_heads + h) * (size_t)max_seq) * DK;
    const bf16_t* kg = kc + head_off;
    const bf16_t* vg = vc + head_off;

    // Q fragments (B operand): lane (j, g) holds Q[query j][32 ks + 8 g ..]
    uint4 qf[2][NDB];
    int qpos[2];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt) {
        const int t = q0 + 16 * jt + j;
        qpos[jt] = (t < T_new) ? S_b + t : -1;  // -1: no such query, every key masked
        const bf16_t* qp = qkv + ((size_t)b * T_new + min(t, T_new - 1)) * (size_t)P * 3 * d_model + (size_t)l * 3 * d_model +
                           (size_t)h * DK + 8 * g;
#pragma unroll
        for (int ks = 0; ks < NDB; ++ks)
            qf[jt][ks] = (t < T_new) ? *reinterpret_cast<const uint4*>(qp + 32 * ks) : make_uint4(0, 0, 0, 0);
    }

    // ---- staging roles.  K: piece p = tid + 256 q -> key p / PPK, piece c = p % PPK of the row.
    // V: group v = tid + 256 q -> d quad dq = v % (DK/4), key group kgp = v / (DK/4): the 8 keys of operand piece
    // (kb2 = kgp >> 2, g = kgp & 3), i.e. key 32 kb2 + 16 (e >> 2) + 4 g + (e & 3) for slot e.
    u32x4 kreg[KPT];  // vector type, not the uint4 struct: struct copies through memcpy kept this array in memory
    uint2 vreg[VG][8];
    auto fetch = [&](int key0) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < KPT; ++q) {
            const int p = tid + kPfThreads * q;
            const int slot = min(key0 + p / PPK, kv_end - 1);  // rows past the end: any row, they are masked
            kreg[q] = *reinterpret_cast<const u32x4*>(kg + (size_t)slot * DK + 8 * (p % PPK));
        }
#pragma unroll
        for (int q = 0; q < VG; ++q) {
            const int v = tid + kPfThreads * q;
            if (v >= NVG) break;
            const int dq = v % (DK / 4), kgp = v / (DK / 4);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = 32 * (kgp >> 2) + 16 * (e >> 2) + 4 * (kgp & 3) + (e & 3);
                const int slot = key0 + key;
                // V rows past the end must be zero: their probabilities are zero, but 0 * garbage may be NaN
                const uint2 raw = *reinterpret_cast<const uint2*>(vg + (size_t)min(slot, kv_end - 1) * DK + 4 * dq);
                const uint32_t keep = slot < kv_end ? 0xffffffffu : 0u;
                vreg[q][e] = make_uint2(raw.x & keep, raw.y & keep);
            }
        }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
        bf16_t* Ks = Ks2 + buf * KSZ;
        bf16_t* Vs = Vs2 + buf * VSZ;
#pragma unroll
        for (int q = 0; q < KPT; ++q) {
            const int p = tid + kPfThreads * q;
            const int key = p / PPK, c = p % PPK;
            const int kt = key >> 4, i = key & 15, db = c >> 2, gg = c & 3;
            const int pos = gg * 16 + ((i + 4 * gg + 2 * (db & 1) + (db >> 1)) & 15);
            *reinterpret_cast<u32x4*>(Ks + (kt * NDB + db) * TE + pos * 8) = kreg[q];
        }
#pragma unroll
        for (int q = 0; q < VG; ++q) {
            const int v = tid + kPfThreads * q;
            if (v >= NVG) break;
            const int dq = v % (DK / 4), kgp = v / (DK / 4);
            const int kb2 = kgp >> 2, gg = kgp & 3, dt = dq >> 2;
#pragma unroll
            for (int dd = 0; dd < 4; ++dd) {
                // piece of d = 4 dq + dd: the 8 keys' values, two per dword
                const uint32_t sel = (dd & 1) ? 0x07060302u : 0x05040100u;
                uint4 o;
                if (dd < 2) {
                    o.x = __builtin_amdgcn_perm(vreg[q][1].x, vreg[q][0].x, sel);
                    o.y = __builtin_amdgcn_perm(vreg[q][3].x, vreg[q][2].x, sel);
                    o.z = __builtin_amdgcn_perm(vreg[q][5].x, vreg[q][4].x, sel);
                    o.w = __builtin_amdgcn_perm(vreg[q][7].x, vreg[q][6].x, sel);
                } else {
                    o.x = __builtin_amdgcn_perm(vreg[q][1].y, vreg[q][0].y, sel);
                    o.y = __builtin_amdgcn_perm(vreg[q][3].y, vreg[q][2].y, sel);
                    o.z = __builtin_amdgcn_perm(vreg[q][5].y, vreg[q][4].y, sel);
                    o.w = __builtin_amdgcn_perm(vreg[q][7].y, vreg[q][6].y, sel);
                }
                const int i = 4 * (dq & 3) + dd;
                // rotate the pieces of a tile by its d tile index: the 16 lanes written together differ in
                // (dq & 3, dt) and then fall into 16 different bank groups
                *reinterpret_cast<uint4*>(Vs + (dt * 2 + kb2) * TE + (gg * 16 + ((i + dt) & 15)) * 8) = o;
            }
        }
    };

    // first query position of the wave (queries past T_new are not stored: they go unmasked and do not count)
    int qmin = min(qpos[0] < 0 ? 0x7fffffff : qpos[0], qpos[1] < 0 ? 0x7fffffff : qpos[1]);
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) qmin = min(qmin, __shfl_xor(qmin, off, kWave));
    qmin = __builtin_amdgcn_readfirstlane(qmin);

    attn_f32x4 acc[NDT][2];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int jt = 0; jt < 2; ++jt) acc[dt][jt] = attn_f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun[2] = {-INFINITY, -INFINITY}, lrun[2] = {0.f, 0.f};
    const float scale2 = 1.4426950408889634f / sqrtf((float)DK);  // scores in units of log 2: exp(x) = exp2(x log2 e)

    // Two LDS stages: while a tile is multiplied, the next one (already in registers) is written to the other
    // stage and the one after that is fetched; one barrier per tile.
    fetch(0);
    stage(0);
    fetch(kPfBKV);  // unconditional: rows past the end are clamped (K) or zero (V)
    __syncthreads();
    for (int key0 = 0, it_tile = 0; key0 < kv_end; key0 += kPfBKV, ++it_tile) {
        const bf16_t* Ks = Ks2 + (it_tile & 1) * KSZ;
        const bf16_t* Vs = Vs2 + (it_tile & 1) * VSZ;

        // ---- S^T = K Q^T for 4 key tiles x 2 query tiles
        attn_f32x4 s[4][2];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
#pragma unroll
            for (int jt = 0; jt < 2; ++jt) s[it][jt] = attn_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NDB; ++ks) {
                const int pos = g * 16 + ((j + 4 * g + 2 * (ks & 1) + (ks >> 1)) & 15);
                const uint4 kf = *reinterpret_cast<const uint4*>(Ks + (it * NDB + ks) * TE + pos * 8);
#pragma unroll
                for (int jt = 0; jt < 2; ++jt)
                    s[it][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(attn_bf16x8, kf),
                                                                        __builtin_bit_cast(attn_bf16x8, qf[jt][ks]), s[it][jt], 0, 0, 0);
            }
        }
        // the other stage was last read before the previous barrier: write the next tile there, fetch the one after
        stage((it_tile & 1) ^ 1);       // after the last tile: a tile of clamped rows that nobody reads
        fetch(key0 + 2 * kPfBKV);
        // ---- mask, online softmax (per query = per column), P fragments
        uint4 pk[2][2];  // [key block][query tile]
        // only tiles that reach past the wave's first query need the causal mask (wave-uniform)
        const bool masked = key0 + kPfBKV - 1 > qmin;
#pragma unroll
        for (int jt = 0; jt < 2; ++jt) {
            // running maximum in raw score units; the scale (log2 e / sqrt(d_k) > 0) enters in the exponent's fma
            float mloc = -INFINITY;
            if (masked) {
#pragma unroll
                for (int it = 0; it < 4; ++it)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int key = key0 + 16 * it + 4 * g + r;
                        const float v = (key <= qpos[jt]) ? s[it][jt][r] : -INFINITY;
                        s[it][jt][r] = v;
                        mloc = fmaxf(mloc, v);
                    }
            } else {
#pragma unroll
                for (int it = 0; it < 4; ++it)
                    mloc = fmaxf(fmaxf(mloc, fmaxf(s[it][jt][0], s[it][jt][1])), fmaxf(s[it][jt][2], s[it][jt][3]));
            }
            mloc = fmaxf(mloc, __shfl_xor(mloc, 16, kWave));
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32, kWave));
            const float mnew = fmaxf(mrun[jt], mloc);
            // exp2(-inf) = 0 covers the first tile and masked keys; a query with no key yet keeps mnew = -inf
            const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
            const float corr = __builtin_amdgcn_exp2f((mrun[jt] - msafe) * scale2);
            const float moff = -msafe * scale2;
            float psum = 0.f;
            float p[4][4];
#pragma unroll
            for (int it = 0; it < 4; ++it)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    p[it][r] = __builtin_amdgcn_exp2f(fmaf(s[it][jt][r], scale2, moff));
                    psum += p[it][r];
                }
            lrun[jt] = lrun[jt] * corr + psum;
            mrun[jt] = mnew;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) {
                acc[dt][jt][0] *= corr; acc[dt][jt][1] *= corr; acc[dt][jt][2] *= corr; acc[dt][jt][3] *= corr;
            }
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2) {
                pk[kb2][jt].x = pack_bf16x2(p[2 * kb2][0], p[2 * kb2][1]);
                pk[kb2][jt].y = pack_bf16x2(p[2 * kb2][2], p[2 * kb2][3]);
                pk[kb2][jt].z = pack_bf16x2(p[2 * kb2 + 1][0], p[2 * kb2 + 1][1]);
                pk[kb2][jt].w = pack_bf16x2(p[2 * kb2 + 1][2], p[2 * kb2 + 1][3]);
            }
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2) {
                const uint4 vf = *reinterpret_cast<const uint4*>(Vs + (dt * 2 + kb2) * TE + (g * 16 + ((j + dt) & 15)) * 8);
#pragma unroll
                for (int jt = 0; jt < 2; ++jt)
                    acc[dt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(attn_bf16x8, vf),
                                                                          __builtin_bit_cast(attn_bf16x8, pk[kb2][jt]), acc[dt][jt], 0, 0, 0);
            }
        __syncthreads();  // this stage is free again, the next one is complete
    }

    // ---- normalise and store: lane (j, g) holds d = 16 dt + 4 g .. + 3 of query j
#pragma unroll
    for (int jt = 0; jt < 2; ++jt) {
        float lt = lrun[jt];
        lt += __shfl_xor(lt, 16, kWave);
        lt += __shfl_xor(lt, 32, kWave);
        const int t = q0 + 16 * jt + j;
        if (t >= T_new) continue;
        const float inv = 1.0f / lt;
        bf16_t* out = ctx + ((size_t)l * M + (size_t)b * T_new + t) * d_model + (size_t)h * DK + 4 * g;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            uint2 o;
            o.x = pack_bf16x2(acc[dt][jt][0] * inv, acc[dt][jt][1] * inv);
            o.y = pack_bf16x2(acc[dt][jt][2] * inv, acc[dt][jt][3] * inv);
            *reinterpret_cast<uint2*>(out + 16 * dt) = o;
        }
    }
}


// ---------------------------------------------------------------------------------------------------------
// The same computation on v_mfma_f32_32x32x16_bf16 (the form that sustains the full matrix rate on gfx950; the
// 16x16x32 form above was measured at 45 to 80 % of it).  Transposed formulation again:
//   S^T[key][query] = K Q^T     A operand = K rows (lane (i, gg): key i of a 32-key tile, d = 16 ks + 8 gg ..),
//                               B operand = Q rows (lane (j, gg): query j)
//   O^T[d][query]   = V^T P^T   A operand = V^T,  B operand = P^T
// A result lane (j, hf) holds rows 8 q + 4 hf + e (register 4 q + e) of column j: 16 keys of one query per 32-key
// tile.  Registers 8 h2 .. 8 h2 + 7 are exactly one B-operand fragment of the second product if the 16 key slots
// (gg, e8) of slab (it, h2) are taken to mean key 32 it + 16 h2 + 8 (e8 >> 2) + 4 gg + (e8 & 3); V^T is staged in
// LDS in that key order, so P never leaves its registers.  The 32 rows of a V^T tile are the d values in the order
// i = 8 (d % 4) + (d / 4) % 8: the four pieces a thread writes after transposing its 8 keys x 4 d block then fall
// next to the pieces of its neighbours (conflict-free 16-byte writes), and a result lane ends up with four
// consecutive d per register quad.  A wave owns 32 queries; its softmax statistics live in the two lanes (j, 0) and
// (j, 1): one cross-lane step.  The accumulator is rescaled only when some query's running maximum moved.
// Workgroup: 4 waves = 128 queries, key tiles of 64, two LDS stages (16 KiB of K, 16 KiB of V^T each for d_k 128).
// ---------------------------------------------------------------------------------------------------------
typedef float attn_f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t attn_u32x2 __attribute__((ext_vector_type(2)));
constexpr uint32_t kAttnBufFlags = 0x00020000u;  // raw buffer, 32-bit data format (the gfx9 / CDNA encoding)

template <int DK>
__global__ __launch_bounds__(kPfThreads, 2) void attn_prefill_mfma32_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc,
    const int32_t* __restrict__ kv_len, bf16_t* __restrict__ ctx, int P, int B, int T_new, int n_heads, int max_seq,
    int b_max) {
    constexpr int NKS = DK / 16;  // k steps of the first product (16 d each)
    constexpr int NDT = DK / 32;  // 32-row d tiles of the second product
    constexpr int PPK = DK / 8;   // 16-byte pieces per key row
    constexpr int TE = 512;       // elements per 1 KiB operand tile (64 pieces)
    constexpr int KPT = (kPfBKV * PPK) / kPfThreads;        // K pieces per thread and tile
    constexpr int NVG = (kPfBKV / 8) * (DK / 4);            // V groups (8 keys x 4 d) of a tile
    static_assert(KPT >= 1 && NVG <= kPfThreads && NVG % 64 == 0, "tile does not fit the workgroup");
    constexpr int KSZ = 2 * NKS * TE, VSZ = NDT * 4 * TE;
    __shared__ __align__(16) bf16_t Ks2[2 * KSZ];   // two stages of [32-key tile 0..1][k step]
    __shared__ __align__(16) bf16_t Vs2[2 * VSZ];   // two stages of [d tile][16-key slab 0..3]

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int j = lane & 31, hf = lane >> 5;
    // workgroup -> (head unit, query block): see the kernel above (a unit's blocks stay on one XCD, longest first)
    const int nqb = (T_new + kPfBQ - 1) / kPfBQ, units = P * B * n_heads;
    const int xcd = blockIdx.x & 7, slot_id = blockIdx.x >> 3;
    const int grp = slot_id / (kPfUnitGroup * nqb), i_in = slot_id % (kPfUnitGroup * nqb);
    const int qb = nqb - 1 - i_in / kPfUnitGroup;
    const int unit = xcd + 8 * (grp * kPfUnitGroup + i_in % kPfUnitGroup);
    if (unit >= units) return;  // padding of the grid (whole workgroup)
    const int h = unit % n_heads;
    const int lb = unit / n_heads;
    const int b = lb % B, l = lb / B;
    const int M = B * T_new;
    const size_t d_model = (size_t)n_heads * DK;
    const int S_b = kv_len[b];
    const int q0 = qb * kPfBQ + 32 * w;
    int kv_end = S_b + min(qb * kPfBQ + kPfBQ, T_new);
    if (kv_end > max_seq) kv_end = max_seq;
    if (kv_end < 1) return;  // a negative kv_len: nothing to read (whole workgroup)
    const size_t head_off = ((((size_t)l * b_max + b) * n_heads + h) * (size_t)max_seq) * DK;
    const bf16_t* kg = kc + head_off;
    const bf16_t* vg = vc + head_off;

    // Q fragments (B operand): lane (j, hf) holds Q[query j][16 ks + 8 hf ..]
    uint4 qf[NKS];
    const int tq = q0 + j;
    const int qpos = (tq < T_new) ? S_b + tq : -1;  // -1: no such query, every key masked
    {
        const bf16_t* qp = qkv + ((size_t)b * T_new + min(tq, T_new - 1)) * (size_t)P * 3 * d_model + (size_t)l * 3 * d_model +
                           (size_t)h * DK + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
            qf[ks] = (tq < T_new) ? *reinterpret_cast<const uint4*>(qp + 16 * ks) : make_uint4(0, 0, 0, 0);
    }

    // ---- staging roles.  K: piece p = tid + 256 q -> key p / PPK, piece c = p % PPK of the row (k step c >> 1,
    // half c & 1); inside its tile the piece goes to slot (key + c) mod 32 of its half, so that the pieces of one
    // row, which neighbouring threads write, fall into different banks.
    // V: group v = tid -> d quad dq = v % (DK/4), key group kgp = v / (DK/4): slab kgp >> 1, half gg = kgp & 1,
    // keys 16 slab + 8 (e8 >> 2) + 4 gg + (e8 & 3).
    u32x4 kreg[KPT];
    uint2 vreg[8];
    const bool v_on = tid < NVG;
    const int v_dq = tid % (DK / 4), v_kgp = (tid / (DK / 4)) & 7;
    // Buffer loads: the descriptor of a tile starts at its first key row and ends at the last valid row, so rows past
    // the end read as zero without any per-lane clamp (K rows there are masked; V rows must be zero: their
    // probabilities are zero, but 0 * garbage may be NaN).  Per-lane byte offsets are fixed for the whole kernel.
    uint32_t k_off[KPT], v_off[8];
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
        const int p = tid + kPfThreads * q;
        k_off[q] = (uint32_t)(((p / PPK) * DK + 8 * (p % PPK)) * 2);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int key = 16 * (v_kgp >> 1) + 8 * (e >> 2) + 4 * (v_kgp & 1) + (e & 3);
        v_off[e] = (uint32_t)((key * DK + 4 * v_dq) * 2);
    }
    auto fetch = [&](int key0) __attribute__((always_inline)) {
        const int rows = max(kv_end - key0, 0);            // wave-uniform
        const uint32_t bytes = (uint32_t)rows * DK * 2;    // at most 64 rows are addressed
        const __amdgpu_buffer_rsrc_t krs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(kg + (size_t)min(key0, kv_end) * DK), 0, bytes, kAttnBufFlags);
        const __amdgpu_buffer_rsrc_t vrs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(vg + (size_t)min(key0, kv_end) * DK), 0, bytes, kAttnBufFlags);
#pragma unroll
        for (int q = 0; q < KPT; ++q)
            kreg[q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(krs, k_off[q], 0, 0));
        if (v_on) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const attn_u32x2 raw = __builtin_amdgcn_raw_buffer_load_b64(vrs, v_off[e], 0, 0);
                vreg[e] = make_uint2(raw[0], raw[1]);
            }
        }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
        bf16_t* Ks = Ks2 + buf * KSZ;
        bf16_t* Vs = Vs2 + buf * VSZ;
#pragma unroll
        for (int q = 0; q < KPT; ++q) {
            const int p = tid + kPfThreads * q;
            const int key = p / PPK, c = p % PPK;
            const int it = key >> 5, i = key & 31, ks = c >> 1, gg = c & 1;
            *reinterpret_cast<u32x4*>(Ks + (it * NKS + ks) * TE + (gg * 32 + ((i + c) & 31)) * 8) = kreg[q];
        }
        if (v_on) {
            const int slab = v_kgp >> 1, gg = v_kgp & 1, dt = v_dq >> 3;
#pragma unroll
            for (int dd = 0; dd < 4; ++dd) {
                // piece of d = 4 dq + dd: the 8 keys' values, two per dword
                const uint32_t sel = (dd & 1) ? 0x07060302u : 0x05040100u;
                uint4 o;
                if (dd < 2) {
                    o.x = __builtin_amdgcn_perm(vreg[1].x, vreg[0].x, sel);
                    o.y = __builtin_amdgcn_perm(vreg[3].x, vreg[2].x, sel);
                    o.z = __builtin_amdgcn_perm(vreg[5].x, vreg[4].x, sel);
                    o.w = __builtin_amdgcn_perm(vreg[7].x, vreg[6].x, sel);
                } else {
                    o.x = __builtin_amdgcn_perm(vreg[1].y, vreg[0].y, sel);
                    o.y = __builtin_amdgcn_perm(vreg[3].y, vreg[2].y, sel);
                    o.z = __builtin_amdgcn_perm(vreg[5].y, vreg[4].y, sel);
                    o.w = __builtin_amdgcn_perm(vreg[7].y, vreg[6].y, sel);
                }
                const int i = 8 * dd + (v_dq & 7);  // row of d = 4 dq + dd inside its 32-d tile
                *reinterpret_cast<uint4*>(Vs + (dt * 4 + slab) * TE + (gg * 32 + i) * 8) = o;
            }
        }
    };

    // first query position of the wave (queries past T_new are not stored: they go unmasked and do not count)
    int qmin = qpos < 0 ? 0x7fffffff : qpos;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) qmin = min(qmin, __shfl_xor(qmin, off, kWave));
    qmin = __builtin_amdgcn_readfirstlane(qmin);

    attn_f32x16 acc[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;
    const float scale2 = 1.4426950408889634f / sqrtf((float)DK);  // scores in units of log 2: exp(x) = exp2(x log2 e)

    fetch(0);
    stage(0);
    fetch(kPfBKV);  // unconditional: rows past the end are clamped (K) or zero (V)
    __syncthreads();
    for (int key0 = 0, it_tile = 0; key0 < kv_end; key0 += kPfBKV, ++it_tile) {
        const bf16_t* Ks = Ks2 + (it_tile & 1) * KSZ;
        const bf16_t* Vs = Vs2 + (it_tile & 1) * VSZ;

        // ---- S^T = K Q^T for two 32-key tiles
        attn_f32x16 s[2];
#pragma unroll
        for (int it = 0; it < 2; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[it][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const uint4 kf = *reinterpret_cast<const uint4*>(Ks + (it * NKS + ks) * TE + (hf * 32 + ((j + 2 * ks + hf) & 31)) * 8);
                s[it] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(attn_bf16x8, kf),
                                                                __builtin_bit_cast(attn_bf16x8, qf[ks]), s[it], 0, 0, 0);
            }
        }
        // the other stage was last read before the previous barrier: write the next tile there, fetch the one after
        stage((it_tile & 1) ^ 1);       // after the last tile: a tile of clamped rows that nobody reads
        fetch(key0 + 2 * kPfBKV);
        // ---- mask, online softmax (per query = per column j: lanes (j, 0) and (j, 1))
        const bool masked = key0 + kPfBKV - 1 > qmin;  // only tiles that reach past the wave's first query (uniform)
        float mloc = -INFINITY;
        if (masked) {
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key0 + 32 * it + 8 * (r >> 2) + 4 * hf + (r & 3);
                    const float v = (key <= qpos) ? s[it][r] : -INFINITY;
                    s[it][r] = v;
                    mloc = fmaxf(mloc, v);
                }
        } else {
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; r += 4)
                    mloc = fmaxf(fmaxf(mloc, fmaxf(s[it][r], s[it][r + 1])), fmaxf(s[it][r + 2], s[it][r + 3]));
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, kWave));
        const float mnew = fmaxf(mrun, mloc);
        // exp2(-inf) = 0 covers the first tile and masked keys; a query with no key yet keeps mnew = -inf
        const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
        const float corr = __builtin_amdgcn_exp2f((mrun - msafe) * scale2);
        const float moff = -msafe * scale2;
        float psum = 0.f;
        uint4 pk[4];  // B-operand fragments of the four 16-key slabs (it, h2)
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            float p[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = __builtin_amdgcn_exp2f(fmaf(s[it][r], scale2, moff));
                psum += p[r];
            }
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                pk[2 * it + h2].x = pack_bf16x2(p[8 * h2 + 0], p[8 * h2 + 1]);
                pk[2 * it + h2].y = pack_bf16x2(p[8 * h2 + 2], p[8 * h2 + 3]);
                pk[2 * it + h2].z = pack_bf16x2(p[8 * h2 + 4], p[8 * h2 + 5]);
                pk[2 * it + h2].w = pack_bf16x2(p[8 * h2 + 6], p[8 * h2 + 7]);
            }
        }
        lrun = lrun * corr + psum;
        mrun = mnew;
        if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {  // some query's maximum moved (wave-uniform branch)
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[dt][r] *= corr;
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                const uint4 vf = *reinterpret_cast<const uint4*>(Vs + (dt * 4 + sl) * TE + (hf * 32 + j) * 8);
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(attn_bf16x8, vf),
                                                                  __builtin_bit_cast(attn_bf16x8, pk[sl]), acc[dt], 0, 0, 0);
            }
        __syncthreads();  // this stage is free again, the next one is complete
    }

    // ---- normalise and store: lane (j, hf), registers e, 4 + e, 8 + e, 12 + e hold d = 32 dt + 16 hf + 4 e .. + 3
    float lt = lrun + __shfl_xor(lrun, 32, kWave);
    if (tq >= T_new) return;
    const float inv = 1.0f / lt;
    bf16_t* out = ctx + ((size_t)l * M + (size_t)b * T_new + tq) * d_model + (size_t)h * DK + 16 * hf;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint2 o;
            o.x = pack_bf16x2(acc[dt][e] * inv, acc[dt][4 + e] * inv);
            o.y = pack_bf16x2(acc[dt][8 + e] * inv, acc[dt][12 + e] * inv);
            *reinterpret_cast<uint2*>(out + 32 * dt + 4 * e) = o;
        }
}

}  // namespace cqil
