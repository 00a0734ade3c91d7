/*
 * cqil.h -- C ABI of the MI355X (gfx950) CQIL library.
 *
 * CQIL = Concurrent Computation of Quasi-Independent Layers (arxiv 2404.06709): a run of P
 * consecutive pre-norm decoder layers is fed one shared hidden state x_G; their attention and
 * feed-forward residual branches are summed into the next shared state (Eq.3), and attention
 * outputs of earlier layers of the group are forwarded into the feed-forward input of later ones
 * ("bypassing", distance d, Eq.4).  The paper places one layer per GPU (Alg.1); this library runs
 * all P layers of a group on ONE GPU as wider kernels over weights packed once per group.
 *
 * General rules
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *  - All work is enqueued on the `stream` argument (a hipStream_t passed as void*; NULL = the
 *    default stream).  No call synchronises, allocates or frees device memory: the caller owns
 *    every buffer (packed weights, KV caches, activations, workspace).
 *  - Return value: CQIL_OK (0) or a negative cqil_status.  Nothing aborts.  Arguments are checked
 *    on the host before anything is launched, so a failed call has enqueued nothing
 *    (except CQIL_EHIP, which reports a launch failure and leaves hipGetLastError() readable).
 *  - A layer is LLaMA-1: bias-free, RMSNorm, rotary embedding with half-split pairing
 *    (element i pairs with i + head_dim/2, angle pos * rope_base^(-2i/head_dim)), multi-head
 *    attention with n_kv_heads == n_heads and a causal mask, SwiGLU feed-forward.  Source weight
 *    matrices are row-major [out, in] (y = W x).
 *  - dtype is the storage type of weights, gains, KV caches and of x_in / x_out; all sums are
 *    accumulated in fp32.
 *  - Thread safety: calls on different streams with disjoint workspaces and KV caches may run
 *    concurrently; a packed group is immutable and may be shared.
 */
#ifndef CQIL_H
#define CQIL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CQIL_OK = 0,
    CQIL_EINVAL = -1, /* null pointer, non-positive size, unsupported shape or dtype */
    CQIL_ESIZE = -2,  /* packed buffer or workspace smaller than the matching *_bytes() query */
    CQIL_ERANGE = -3, /* max_kv_len + T exceeds max_seq, or B exceeds b_max */
    CQIL_EHIP = -4    /* a kernel launch failed */
} cqil_status;

typedef enum { CQIL_F32 = 0, CQIL_BF16 = 1 } cqil_dtype;

/* Value of bypass_d that selects the attention-FFN parallel form (App. A, Eq.5) instead of Eq.4. */
#define CQIL_ATTN_FFN_PARALLEL (-1)

/* Shape of one decoder layer.  Requirements: n_heads * head_dim == d_model; head_dim a power of two,
 * 32..256; d_model % 32 == 0, at most 14336; d_ffn % 16 == 0; max_seq >= 1. */
typedef struct {
    int d_model, n_heads, head_dim, d_ffn, max_seq;
    float rope_base, rms_eps;
    int dtype; /* cqil_dtype */
} cqil_dims;

/* Source weights of one layer (Eq.2's W^Q, W^K, W^V, W^O; W_1 split into gate and up, W_2 = down). */
typedef struct {
    const void *wq, *wk, *wv, *wo; /* [d_model, d_model] */
    const void *wgate, *wup;       /* [d_ffn, d_model] */
    const void *wdown;             /* [d_model, d_ffn] */
    const void *g_attn, *g_ffn;    /* [d_model] RMSNorm gains of the attention / feed-forward module */
} cqil_layer;

/* KV caches of one group: every layer keeps its own cache, filled from the SHARED input x_G
 * (consequence of ATTN_l(x_G) in Eq.3).  Layout [P][b_max][n_heads][max_seq][head_dim], dtype;
 * K is stored after the rotary embedding.  A call touches only slots kv_len[b] .. kv_len[b]+T-1
 * of sequences b < B; every other byte is preserved bit for bit. */
typedef struct {
    void *k, *v;
    int32_t *kv_len; /* [b_max] tokens already cached per sequence; the same for all P layers */
    int b_max;
    int max_kv_len;  /* host-side upper bound of kv_len[b] before the call, used only for the host's range
                        check max_kv_len + T <= max_seq (kernels read the exact lengths from kv_len and
                        never write past max_seq even if this bound is wrong).  Advanced with kv_len. */
} cqil_kv;

/* Byte offsets of the parts of a packed group (all multiples of 256).  Logical matrices:
 *   wqkv   [P*3*d_model][d_model]   rows of Wq, Wk, Wv of layer 0, then of layer 1, ...        (N-concat)
 *   wo     [d_model][P*d_model]     row o = the P layers' rows o of Wo side by side             (K-concat)
 *   wgu    [P*2*d_ffn][d_model]     per layer: 16 rows of Wgate, the matching 16 rows of Wup,
 *                                   the next 16 rows of Wgate, ...                              (N-concat)
 *   wdown  [d_model][P*d_ffn]       row o = the P layers' rows o of Wdown side by side          (K-concat)
 * With the K-concatenated layouts the sums over layers in Eq.3 / Eq.4 are part of the contraction.
 * Each logical matrix W[R][K] is stored in 1 KiB tiles of 16 rows x KB columns, KB = 64 / sizeof(element)
 * (32 for bf16, 16 for fp32); K is padded with zero columns to a multiple of KB (Kp).  The tiles of one 16-row
 * strip follow each other along k; inside a tile the 16-byte pieces are ordered [g][i], piece (g, i) holding
 * columns KB*kb + (KB/4)*g .. + KB/4 - 1 of row 16*rt + i.  Element (r, k) therefore sits at element offset
 *   ((r/16)*(Kp/KB) + k/KB)*16*KB + ((k%KB)/(KB/4))*16*(KB/4) + (r%16)*(KB/4) + k%(KB/4).
 * A 64-lane wave reads one tile with one contiguous 16-byte load per lane, and lane i + 16 g receives its
 * fragment (row i, k group g) of the A operand of the 16x16x32 bf16 matrix-core instruction.
 *   g_attn, g_ffn [P][d_model]
 *   rope   [max_seq][head_dim/2] pairs (cos, sin) of pos * rope_base^(-2i/head_dim), fp32,
 *          evaluated in double and rounded once */
typedef struct {
    size_t wqkv, wo, wgu, wdown, g_attn, g_ffn, rope, total;
} cqil_packed_layout;

const char *cqil_strerror(int status);

/* host-only: checks dims and P (1..16) and fills the layout; no GPU needed */
int cqil_packed_layout_of(const cqil_dims *dims, int P, cqil_packed_layout *out /* host */);
/* 0 if the arguments are invalid */
size_t cqil_packed_bytes(const cqil_dims *dims, int P);
size_t cqil_workspace_bytes(const cqil_dims *dims, int P, int B, int T);
/* Testing aid: after cqil_group_forward has run, the workspace holds the attention outputs
 * attn_i = ATTN_i(x) of Eq.3 / Eq.4 as fp32 [P][B*T][d_model] at this byte offset ((size_t)-1 if the
 * arguments are invalid).  Nothing else about the workspace contents is specified. */
size_t cqil_workspace_attn_out_offset(const cqil_dims *dims, int P, int B, int T);

/* Sec.4.2 partition rule, host-only: layers s..e (1-indexed, inclusive) form consecutive groups of
 * at most p layers, every other layer is a group of one.  group_sizes_out (host) needs room for L
 * ints.  Example from the paper: L=32, p=2, s=9, e=30 -> 8 singles, 11 pairs, 2 singles. */
int cqil_partition(int L, int p, int s, int e, int *group_sizes_out, int *n_groups_out);

/* One-time packing of P layers into `packed` (cqil_packed_bytes() bytes, 256-byte aligned).
 * Pure data movement for the weights (bit-exact copies at the documented indices) plus the rotary
 * table.  layers: host array of P structs holding device pointers. */
int cqil_pack_group(const cqil_dims *dims, int P, const cqil_layer *layers /* host */, void *packed,
                    size_t packed_bytes, void *stream);

/* Folds a LoRA adapter into a source weight matrix before packing (Sec.5.1, App. C: the paper fine-tunes
 * adapters on every linear matrix of the attention and feed-forward modules with alpha = rank, i.e. scale 1):
 *   W[o][k] += scale * sum_j Bm[o][j] * A[j][k]
 * W [n_out][n_in] (device, row-major, updated in place), A [rank][n_in], Bm [n_out][rank], all of `dtype`
 * (cqil_dtype); fp32 accumulation and one rounding to dtype.  n_in must be a multiple of 16 / sizeof(dtype),
 * 1 <= rank <= 1024, W and A 16-byte aligned; otherwise CQIL_EINVAL.  Asynchronous on `stream`. */
int cqil_merge_lora(void *W, const void *A, const void *Bm, int dtype, int n_out, int n_in, int rank, float scale,
                    void *stream);

/* Similarity of layer inputs (Sec.3.1, the measurement that motivates which layers to group): X (device)
 * [L][M][n] of `dtype` holds the inputs x_l of L layers for the same M tokens (captured by the caller, e.g. by
 * running the model as groups of one); sim (device, fp32 [L][L]) receives the mean over tokens of the per-token
 * cosine <x_a, x_b> / (|x_a| |x_b|) (0 for a zero vector).  workspace: cqil_input_similarity_workspace_bytes(L, M)
 * bytes (0 for invalid arguments).  1 <= L <= 1024, n a multiple of 16 / sizeof(dtype), X 16-byte aligned;
 * otherwise CQIL_EINVAL; a short workspace is CQIL_ESIZE.  Deterministic; asynchronous on `stream`. */
size_t cqil_input_similarity_workspace_bytes(int L, int M);
int cqil_input_similarity(const void *X, int dtype, int L, int M, int n, float *sim, void *workspace,
                          size_t workspace_bytes, void *stream);

/* One group step (Eq.4; Eq.3 when bypass_d == 0; Eq.1 when P == 1):
 *   attn_i = ATTN_i(x)                                   i = 0..P-1, all from the same x
 *   h_i    = x + attn_i + sum_{j : 1 <= i-j <= d} attn_j
 *   x_out  = x + sum_i attn_i + sum_i FFN_i(h_i)
 * x_in, x_out: [B][T][d_model] dtype; x_out may alias x_in.  T == 1 is a decode step, T > 1 a
 * prefill chunk at positions kv_len[b] .. kv_len[b]+T-1 (causal over cache + new tokens).
 * bypass_d >= P acts as P-1; bypass_d == CQIL_ATTN_FFN_PARALLEL (-1) selects the attention-FFN parallel form
 * of App. A (Eq.5) for every layer of the group: each feed-forward module reads x itself,
 * x_out = x + sum_l ATTN_l(x) + sum_l FFN_l(x); any other negative value is CQIL_EINVAL.  advance_kv_len != 0 adds T to
 * kv_len[b] (b < B) and to kv->max_kv_len after the step. workspace: cqil_workspace_bytes()
 * bytes, 256-byte aligned, contents undefined on entry and exit. */
int cqil_group_forward(const cqil_dims *dims, int P, int bypass_d, const void *packed, cqil_kv *kv /* host */,
                       const void *x_in, void *x_out, int B, int T, int advance_kv_len, void *workspace,
                       size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): cqil_group_forward with the workspace in a static device array
 * of cqil_static_scratch_bytes() bytes (8 MiB) that is part of the library's code object; every GPU the library
 * runs on holds its own copy until the process ends.  Same arguments, results and error returns as
 * cqil_group_forward, bit for bit (the same kernels run); a step whose cqil_workspace_bytes() exceeds the array
 * (long prefill chunks, wide batches) is CQIL_ESIZE.  Single-token decode of a 33B-shaped group of up to 16 layers
 * fits.  The call allocates nothing, frees nothing and does not synchronise; its first call on a device looks up
 * the array's address (CQIL_EHIP if that fails).  All calls on one GPU share that GPU's array: calls that may
 * overlap in time on one GPU (different streams, different threads) race; serialise them on one stream. */
size_t cqil_static_scratch_bytes(void);
int cqil_group_forward_static(const cqil_dims *dims, int P, int bypass_d, const void *packed, cqil_kv *kv /* host */,
                              const void *x_in, void *x_out, int B, int T, int advance_kv_len, void *stream);

/* Measurement aid for a single-token decode step (B must be 1, T == 1, kv_len not advanced): the same six
 * kernels as cqil_group_forward, with HIP events recorded on `stream` around each of them.  Waits for the
 * step to finish and writes the six elapsed times in milliseconds to kernel_ms_out (host, 6 floats), in
 * the order: QKV projection (+norm, rotary, append), attention, O projection, gate/up (+bypass, norm,
 * SwiGLU), down projection, merge of Eq.3 / Eq.4.  In the fused schedule of bypass_d == -1 (see cqil_set_tuning,
 * "eq5_fused") slot 0 holds the QKV + gate/up launch, slot 2 the O + down launch, slots 3 and 4 are zero.
 * Creates and destroys its events; blocks the host. */
int cqil_decode_step_profile(const cqil_dims *dims, int P, int bypass_d, const void *packed, cqil_kv *kv /* host */,
                             const void *x_in, void *x_out, int B, void *workspace, size_t workspace_bytes,
                             void *stream, float *kernel_ms_out /* host */);

/* Measurement aid: one kernel that reads buf[0 .. bytes) (bytes a multiple of 16, buf 16-byte aligned) exactly once
 * with the streaming loads the decode kernels use for weights, and writes a checksum per workgroup to sink (device,
 * at least 16384 bytes, 4-byte aligned; CQIL_ESIZE if sink_bytes is smaller).  Timed by the caller, it gives the
 * read-only stream rate of this GPU: the practical ceiling of the bandwidth-bound kernels.  Asynchronous. */
int cqil_stream_read_probe(const void *buf, size_t bytes, void *sink, size_t sink_bytes, void *stream);

/* Whole model (Alg.1 around LLaMA's embedding, final RMSNorm and lm head). */
typedef struct {
    cqil_dims dims;
    int vocab;
    int n_groups;
    const int *group_sizes;     /* host [n_groups], from cqil_partition */
    const void *const *packed;  /* host [n_groups] of device pointers, one packed group each */
    void *const *k_cache;       /* host [n_groups] of device pointers, [P_g][b_max][n][max_seq][head_dim] */
    void *const *v_cache;       /* host [n_groups] */
    int32_t *kv_len;            /* device [b_max], shared by all layers */
    int b_max;
    int max_kv_len;             /* host-side bound, see cqil_kv */
    const void *embedding;      /* [vocab][d_model] dtype */
    const void *g_final;        /* [d_model] */
    const void *lm_head;        /* [vocab][d_model] */
} cqil_model;

size_t cqil_model_workspace_bytes(const cqil_model *m /* host */, int B, int T);

/* tokens [B][T] int32 (device; an id outside 0 .. vocab-1 is clamped to that range by the embedding gather, never
 * read out of the table) -> groups in order -> final norm of the last position -> logits -> greedy token
 * (lowest index among equal maxima).  hidden_out (optional) [B][T][d_model] dtype is the state after
 * the last layer; logits_out (optional) [B][vocab] fp32; next_token_out (optional) [B] int32.
 * kv_len and m->max_kv_len advance by T when advance_kv_len != 0. */
int cqil_model_forward(cqil_model *m /* host */, const int32_t *tokens, int B, int T, int bypass_d,
                       int advance_kv_len, void *hidden_out, float *logits_out, int32_t *next_token_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Input substitution (Sec.3.2, the sensitivity study that decides which layers may share an input): the model runs
 * as cqil_model_forward does, except that group `group` (0-based index into group_sizes; a layer when every group has
 * one layer, as in the paper's experiment) reads the input of group `group - k` instead of its own:
 *   x_after = x_before + F_group(x_input_of(group - k)),   F = the group's attention and feed-forward branches,
 * every other term unchanged, later groups see the changed state.  Its KV cache is filled from the substituted input.
 * k == 0 is cqil_model_forward; 0 <= k <= group < n_groups, else CQIL_EINVAL.  workspace:
 * cqil_model_substituted_workspace_bytes() bytes (one more hidden state than the plain model loop). */
size_t cqil_model_substituted_workspace_bytes(const cqil_model *m /* host */, int B, int T);
int cqil_model_forward_substituted(cqil_model *m /* host */, const int32_t *tokens, int B, int T, int bypass_d,
                                   int advance_kv_len, int group, int k, void *hidden_out, float *logits_out,
                                   int32_t *next_token_out, void *workspace, size_t workspace_bytes, void *stream);

/* Launch-shape knobs (process-wide, host-only, not thread-safe; set them
 * before sizing workspaces).  Keys: "ksplit_qkv", "ksplit_o", "ksplit_gu", "ksplit_d" (waves that share one unit
 * of work and split its k range in the QKV / O / gate-up / down kernel: 1, 2, 4 or 8; 0 = chosen by shape),
 * "down_slice_max" (longest K slice of the down projection, multiple of 512, at
 * most 12288; default 3072): single-token decode kernels.  "gemm_tile" (workgroup tile of the bf16 matrix-core GEMM of the
 * token-parallel path: 1 = 256 tokens x 256 weight rows, 2 = 128 x 256 and the tiled kernel also for up to 8 token
 * rows, where the default is a barrier-free streaming kernel; 0 = default).  The k split, the number of K slices and,
 * for up to 8 rows, the choice between the two GEMM kernels change the order in which partial sums are added, nothing
 * else; for more rows the GEMM tile changes no result at all.  "attn_prefill" (matrix-core attention of bf16 prefill chunks: 0 = default, the kernel built on 32x32x16
 * instructions; 1 = the kernel built on 16x16x32 instructions; same arithmetic, different order of partial sums).
 * "eq5_fused" (single-token step of the attention-FFN parallel
 * form, bypass_d == -1: 1 = default, the step runs as three fused phases -- QKV and gate/up as one shared-input
 * launch, attention, O and down as one K-concatenated launch -- plus the merge; 0 = the six-kernel schedule of Eq.4;
 * both give the same result bit for bit).  Unknown key or bad value: CQIL_EINVAL. */
int cqil_set_tuning(const char *key, int value);

/* Library build information (host-only). */
const char *cqil_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CQIL_H */
