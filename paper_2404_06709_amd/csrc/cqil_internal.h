// Host-side internals of libcqil: buffer layouts and kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/cqil.h"

namespace cqil {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }
inline size_t esize(int dtype) { return dtype == CQIL_BF16 ? 2 : 4; }

constexpr int kGuBlock = 16;        // gate/up rows are interleaved in blocks of this many rows
constexpr int kMaxP = 16;

// Launch-shape knobs of the single-token decode kernels (cqil_set_tuning): waves that share one unit of work
// (k split: 1, 2, 4 or 8; 0 = chosen by shape) in the QKV, O, gate/up and down kernels, and the longest K slice of the down projection
// (multiple of 512, at most 12288).  gemm_tile: workgroup tile of the matrix-core GEMM of the token-parallel path
// (1 = 256 tokens x 256 weight rows, 2 = 128 x 256; 0 = default).
// Atomics: a knob may be set while another thread launches (each launch reads a knob once; a step sized with one
// value of down_slice_max and launched with another is caught by the workspace-size check or runs with the new one).
struct Tuning {
    std::atomic<int> ksplit_qkv{0}, ksplit_o{0}, ksplit_gu{0}, ksplit_d{0}, down_slice_max{3072};  // 0 = by shape
    std::atomic<int> gemm_tile{0};
    std::atomic<int> attn_prefill{0};  // matrix-core prefill attention: 0 = 32x32x16 instructions, 1 = 16x16x32
    std::atomic<int> eq5_fused{1};  // single-token Eq.5 step: 1 = three fused phases, 0 = the six-kernel schedule
};
extern Tuning g_tune;

// Workspace of one group step.  Offsets in bytes, all multiples of 256.
struct WsLayout {
    // decode fast path (B*T == 1) and shared
    size_t q;          // f32 [P][M][d_model]     rotated queries
    size_t ctx;        // f32 [P][M][d_model]     attention context (heads concatenated)
    size_t a;          // f32 [P][M][d_model]     attention outputs a_i
    size_t u;          // f32 [P*d_ffn] (single token): SwiGLU outputs
    size_t down_part;  // f32 [slices][d_model] split-K partials of the single-token down projection
    // token-parallel path (M = B*T > 1); act = dtype of the call
    size_t nrm;        // act [P][M][d_model]     normalised inputs (attention norm, later FFN norm)
    size_t qkv;        // act [M][P*3*d_model]
    size_t ctx_act;    // act [P][M][d_model]
    size_t resid;      // f32 [M][d_model]        x + sum_i a_i
    size_t gu;         // act [M][P*2*d_ffn]
    size_t u_act;      // act [M][P*d_ffn]
    size_t gemm_part;  // f32 split-K partial sums of the matrix-core GEMM (bf16, M <= 512), gemm_part_floats long
    size_t gemm_part_floats;
    size_t total;
    int n_slices, down_slice;  // K slices of the single-token down projection
};

int check_dims(const cqil_dims* d, int P);
int ws_layout(const cqil_dims* d, int P, int B, int T, WsLayout* out);

struct PackArgs {
    cqil_layer layers[kMaxP];
};

// launchers; every one returns a hipError_t from the launch
hipError_t launch_pack(const cqil_dims& d, int P, const PackArgs& src, char* packed, const cqil_packed_layout& L,
                       hipStream_t st);

hipError_t launch_merge_lora(void* W, const void* A, const void* Bm, int dtype, int n_out, int n_in, int r, float scale,
                             hipStream_t st);

hipError_t launch_similarity(const void* X, int dtype, int L, int M, int n, float* sim, float* part, int chunks,
                             int tokens_per_chunk, hipStream_t st);

constexpr int kStreamProbeWorkgroups = 4096;  // sink of cqil_stream_read_probe: this many uint32
hipError_t launch_stream_read(const void* buf, size_t bytes, uint32_t* sink, int workgroups, hipStream_t st);

struct StepArgs {
    cqil_dims d;
    int P, bypass_d, B, T, advance;
    const char* packed;
    cqil_packed_layout pl;
    void *kc, *vc;
    int32_t* kv_len;
    int b_max, max_kv_len;
    const void* x_in;
    const void* x_res;  // state the branches are added to (x_in itself, or another state under input substitution)
    void* x_out;
    char* ws;
    WsLayout wl;
    hipEvent_t* ev;  // null, or 7 events recorded around the six decode kernels
};

hipError_t launch_decode_step(const StepArgs& a, hipStream_t st);   // B*T == 1
hipError_t launch_generic_step(const StepArgs& a, hipStream_t st);  // any B, T

struct HeadArgs {
    cqil_dims d;
    int vocab, B, T;
    const void* hidden;   // act [B][T][d_model]
    const void* g_final;  // [d_model]
    const void* lm_head;  // [vocab][d_model]
    float* logits;        // [B][vocab] (workspace if the caller passed none)
    int32_t* next_token;  // [B] or null
    char* ws;             // scratch for the argmax partials
};
hipError_t launch_embedding(const cqil_dims& d, const void* emb, const int32_t* tokens, int M, int vocab, void* x,
                            hipStream_t st);
hipError_t launch_head(const HeadArgs& a, hipStream_t st);
hipError_t launch_advance(int32_t* kv_len, int B, int T, hipStream_t st);
hipError_t launch_copy16(const void* src, void* dst, size_t bytes, hipStream_t st);  // bytes % 16 == 0

}  // namespace cqil
