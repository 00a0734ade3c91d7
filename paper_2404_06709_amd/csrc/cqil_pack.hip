// cqil_pack_group: one-time packing of P layers' weights into the group layout.
//
// The paper places layer l+i of a group on GPU i (Alg.1).  On one GPU the same independence is
// expressed by concatenation: projections that read the shared input (Wq, Wk, Wv; Wgate, Wup) are
// stacked along their output dimension, and the projections whose results Eq.3 / Eq.4 sum over the
// group (Wo, Wdown) are laid side by side along their input dimension, so that the sum over layers is
// part of one long dot product.  Everything here is a pure index map on 16-byte vectors.
#include "cqil_dev.h"
#include "cqil_internal.h"

namespace cqil {

struct PackPtrs {
    const char* p[kMaxP];
};

// dst[(l*3 + m)][o][:] = W_m of layer l, row o          (m = 0,1,2 for q,k,v)
__global__ void pack_qkv_kernel(PackPtrs wq, PackPtrs wk, PackPtrs wv, uint4* dst, int P, int d_model, int vec_per_row) {
    const size_t per_mat = (size_t)d_model * vec_per_row;
    const size_t total = per_mat * 3 * (size_t)P;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t mat = i / per_mat, within = i - mat * per_mat;
        const int l = (int)(mat / 3), m = (int)(mat % 3);
        const char* src = m == 0 ? wq.p[l] : (m == 1 ? wk.p[l] : wv.p[l]);
        dst[i] = reinterpret_cast<const uint4*>(src)[within];
    }
}

// dst[o][l][:] = W of layer l, row o   (rows of `cols` elements; used for Wo and Wdown)
__global__ void pack_kcat_kernel(PackPtrs w, uint4* dst, int P, int rows, int vec_per_row) {
    const size_t total = (size_t)rows * P * vec_per_row;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t v = i % vec_per_row;
        const size_t ol = i / vec_per_row;
        const int l = (int)(ol % P);
        const size_t o = ol / P;
        dst[i] = reinterpret_cast<const uint4*>(w.p[l])[o * vec_per_row + v];
    }
}

// dst[l][j/16][gu][j%16][:] = (gu ? Wup : Wgate) of layer l, row j
__global__ void pack_gu_kernel(PackPtrs wg, PackPtrs wu, uint4* dst, int P, int d_ffn, int vec_per_row) {
    const size_t total = (size_t)P * 2 * d_ffn * vec_per_row;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t v = i % vec_per_row;
        size_t r = i / vec_per_row;  // packed row
        const int l = (int)(r / (2 * (size_t)d_ffn));
        r -= (size_t)l * 2 * d_ffn;
        const int blk = (int)(r / (2 * kGuBlock));
        const int in = (int)(r % (2 * kGuBlock));
        const int gu = in / kGuBlock;
        const int j = blk * kGuBlock + in % kGuBlock;
        const char* src = gu ? wu.p[l] : wg.p[l];
        dst[i] = reinterpret_cast<const uint4*>(src)[(size_t)j * vec_per_row + v];
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

hipError_t launch_pack(const cqil_dims& d, int P, const PackArgs& src, char* packed, const cqil_packed_layout& L,
                       hipStream_t st) {
    const int es = (int)esize(d.dtype);
    const int vpr_dm = d.d_model * es / 16;  // 16-byte vectors per row of d_model elements
    const int vpr_f = d.d_ffn * es / 16;
    PackPtrs a, b, c;
    const int T = 256;

    for (int l = 0; l < P; ++l) { a.p[l] = (const char*)src.layers[l].wq; b.p[l] = (const char*)src.layers[l].wk; c.p[l] = (const char*)src.layers[l].wv; }
    hipLaunchKernelGGL(pack_qkv_kernel, dim3(grid_for((size_t)P * 3 * d.d_model * vpr_dm, T)), dim3(T), 0, st, a, b, c,
                       (uint4*)(packed + L.wqkv), P, d.d_model, vpr_dm);

    for (int l = 0; l < P; ++l) a.p[l] = (const char*)src.layers[l].wo;
    hipLaunchKernelGGL(pack_kcat_kernel, dim3(grid_for((size_t)P * d.d_model * vpr_dm, T)), dim3(T), 0, st, a,
                       (uint4*)(packed + L.wo), P, d.d_model, vpr_dm);

    for (int l = 0; l < P; ++l) { a.p[l] = (const char*)src.layers[l].wgate; b.p[l] = (const char*)src.layers[l].wup; }
    hipLaunchKernelGGL(pack_gu_kernel, dim3(grid_for((size_t)P * 2 * d.d_ffn * vpr_dm, T)), dim3(T), 0, st, a, b,
                       (uint4*)(packed + L.wgu), P, d.d_ffn, vpr_dm);

    for (int l = 0; l < P; ++l) a.p[l] = (const char*)src.layers[l].wdown;
    hipLaunchKernelGGL(pack_kcat_kernel, dim3(grid_for((size_t)P * d.d_model * vpr_f, T)), dim3(T), 0, st, a,
                       (uint4*)(packed + L.wdown), P, d.d_model, vpr_f);

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

}  // namespace cqil
