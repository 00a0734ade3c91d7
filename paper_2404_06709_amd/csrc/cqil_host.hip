// C ABI of libcqil: argument checking, buffer layouts, the (p, s, e) partition and the model-level loop.
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "cqil_internal.h"

namespace cqil {

Tuning g_tune;

static bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int check_dims(const cqil_dims* d, int P) {
    if (!d) return CQIL_EINVAL;
    if (P < 1 || P > kMaxP) return CQIL_EINVAL;
    if (d->dtype != CQIL_F32 && d->dtype != CQIL_BF16) return CQIL_EINVAL;
    if (d->d_model < 32 || d->n_heads < 1 || d->head_dim < 32 || d->d_ffn < 16 || d->max_seq < 1) return CQIL_EINVAL;
    if ((long long)d->n_heads * d->head_dim != d->d_model) return CQIL_EINVAL;
    if (d->d_model % 32 || d->d_ffn % kGuBlock) return CQIL_EINVAL;  // whole tiles of the packed layout
    if (d->d_model > 14336) return CQIL_EINVAL;  // the normalised input of a projection sits in LDS as fp32
    // lanes sharing one cache slot in the attention kernels: head_dim * esize / 16 must be 4, 8, 16, 32 or 64
    const int lps = d->head_dim * (int)esize(d->dtype) / 16;
    if (!pow2(d->head_dim) || lps < 4 || lps > 64) return CQIL_EINVAL;
    if (!(d->rope_base > 1.0f) || !(d->rms_eps >= 0.0f)) return CQIL_EINVAL;
    return CQIL_OK;
}

static int packed_layout(const cqil_dims* d, int P, cqil_packed_layout* L) {
    int rc = check_dims(d, P);
    if (rc) return rc;
    if (!L) return CQIL_EINVAL;
    const size_t es = esize(d->dtype), dm = d->d_model, f = d->d_ffn;
    size_t off = 0;
    L->wqkv = off;   off = align_up(off + (size_t)P * 3 * dm * dm * es);
    L->wo = off;     off = align_up(off + (size_t)P * dm * dm * es);
    L->wgu = off;    off = align_up(off + (size_t)P * 2 * f * dm * es);
    const size_t kb = 64 / es;  // columns per tile; the concatenated K of Wdown is padded to whole tiles
    const size_t kp_down = ((size_t)P * f + kb - 1) / kb * kb;
    L->wdown = off;  off = align_up(off + dm * kp_down * es);
    L->g_attn = off; off = align_up(off + (size_t)P * dm * es);
    L->g_ffn = off;  off = align_up(off + (size_t)P * dm * es);
    L->rope = off;   off = align_up(off + (size_t)d->max_seq * (d->head_dim / 2) * 2 * sizeof(float));
    L->total = off;
    return CQIL_OK;
}

int ws_layout(const cqil_dims* d, int P, int B, int T, WsLayout* W) {
    int rc = check_dims(d, P);
    if (rc) return rc;
    if (B < 1 || T < 1 || !W) return CQIL_EINVAL;
    if ((long long)B * T > (1ll << 24)) return CQIL_EINVAL;
    const size_t M = (size_t)B * T, dm = d->d_model, f = d->d_ffn, es = esize(d->dtype);
    memset(W, 0, sizeof(*W));
    const size_t K = (size_t)P * f;
    const size_t ktile = 64 / es;
    const size_t Kp = (K + ktile - 1) / ktile * ktile;  // padded K of the packed Wdown (whole tiles)
    // K slices of the decode down projection: equal lengths, multiples of 512, at most the tuned maximum
    const size_t smax = (size_t)g_tune.down_slice_max.load();
    int ns = (int)((Kp + smax - 1) / smax);
    size_t sl = ((Kp + ns - 1) / ns + 511) / 512 * 512;
    ns = (int)((Kp + sl - 1) / sl);
    W->n_slices = ns;
    W->down_slice = (int)sl;
    size_t off = 0;
    W->q = off;         off = align_up(off + (size_t)P * M * dm * sizeof(float));
    W->ctx = off;       off = align_up(off + (size_t)P * M * dm * sizeof(float));
    W->a = off;         off = align_up(off + (size_t)P * M * dm * sizeof(float));
    if (M == 1) {
        W->u = off;         off = align_up(off + K * sizeof(float));
        W->down_part = off; off = align_up(off + (size_t)ns * dm * sizeof(float));
    } else {
        W->nrm = off;     off = align_up(off + (size_t)P * M * dm * es);
        W->qkv = off;     off = align_up(off + M * (size_t)P * 3 * dm * es);
        W->ctx_act = off; off = align_up(off + (size_t)P * M * dm * es);
        W->resid = off;   off = align_up(off + M * dm * sizeof(float));
        W->gu = off;      off = align_up(off + M * (size_t)P * 2 * f * es);
        W->u_act = off;   off = align_up(off + M * K * es);
        if (d->dtype == CQIL_BF16 && M <= 512) {
            // up to 16 K slices of the widest product (P groups of M x d_model), capped at 128 MiB
            size_t pf = (size_t)16 * P * M * dm;
            if (pf > ((size_t)32 << 20)) pf = (size_t)32 << 20;
            W->gemm_part = off;
            W->gemm_part_floats = pf;
            off = align_up(off + pf * sizeof(float));
        }
    }
    W->total = off;
    return CQIL_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Workspace of cqil_group_forward_static: one array per GPU, part of the loaded code object, held until the process
// ends.  Host code never passes the array's name to a kernel (on the host the name is only a handle of the symbol):
// the device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices];

// device address of this GPU's copy of `scratch` (looked up on the first call with that device current)
static int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CQIL_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CQIL_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CQIL_OK;
}

}  // namespace cqil

using namespace cqil;

extern "C" {

const char* cqil_version(void) { return "cqil-mi355x 0.1 (gfx950)"; }

const char* cqil_strerror(int status) {
    switch (status) {
        case CQIL_OK: return "ok";
        case CQIL_EINVAL: return "invalid argument";
        case CQIL_ESIZE: return "buffer too small";
        case CQIL_ERANGE: return "sequence or batch out of range";
        case CQIL_EHIP: return "HIP launch failure";
        default: return "unknown status";
    }
}

int cqil_set_tuning(const char* key, int value) {
    if (!key) return CQIL_EINVAL;
    const bool split_ok = value == 0 || value == 1 || value == 2 || value == 4 || value == 8;  // 0 = by shape
    if (!strcmp(key, "ksplit_qkv")) {
        if (!split_ok) return CQIL_EINVAL;
        g_tune.ksplit_qkv = value;
    } else if (!strcmp(key, "ksplit_o")) {
        if (!split_ok) return CQIL_EINVAL;
        g_tune.ksplit_o = value;
    } else if (!strcmp(key, "ksplit_gu")) {
        if (!split_ok) return CQIL_EINVAL;
        g_tune.ksplit_gu = value;
    } else if (!strcmp(key, "ksplit_d")) {
        if (!split_ok) return CQIL_EINVAL;
        g_tune.ksplit_d = value;
    } else if (!strcmp(key, "down_slice_max")) {
        if (value < 512 || value > 12288 || value % 512) return CQIL_EINVAL;
        g_tune.down_slice_max = value;
    } else if (!strcmp(key, "gemm_tile")) {
        if (value < 0 || value > 2) return CQIL_EINVAL;
        g_tune.gemm_tile = value;
    } else if (!strcmp(key, "attn_prefill")) {
        if (value < 0 || value > 1) return CQIL_EINVAL;
        g_tune.attn_prefill = value;
    } else if (!strcmp(key, "eq5_fused")) {
        if (value < 0 || value > 1) return CQIL_EINVAL;
        g_tune.eq5_fused = value;
    } else {
        return CQIL_EINVAL;
    }
    return CQIL_OK;
}

int cqil_packed_layout_of(const cqil_dims* dims, int P, cqil_packed_layout* out) { return packed_layout(dims, P, out); }

size_t cqil_packed_bytes(const cqil_dims* dims, int P) {
    cqil_packed_layout L;
    return packed_layout(dims, P, &L) ? 0 : L.total;
}

size_t cqil_workspace_bytes(const cqil_dims* dims, int P, int B, int T) {
    WsLayout W;
    return ws_layout(dims, P, B, T, &W) ? 0 : W.total;
}

size_t cqil_workspace_attn_out_offset(const cqil_dims* dims, int P, int B, int T) {
    WsLayout W;
    return ws_layout(dims, P, B, T, &W) ? (size_t)-1 : W.a;
}

int cqil_partition(int L, int p, int s, int e, int* group_sizes_out, int* n_groups_out) {
    if (!group_sizes_out || !n_groups_out) return CQIL_EINVAL;
    if (L < 1 || p < 1 || s < 1 || e > L || s > e + 1) return CQIL_EINVAL;
    int n = 0;
    for (int l = 1; l <= L;) {
        int sz = 1;
        if (l >= s && l <= e) {
            const int left = e - l + 1;
            sz = left < p ? left : p;
        }
        group_sizes_out[n++] = sz;
        l += sz;
    }
    *n_groups_out = n;
    return CQIL_OK;
}

int cqil_pack_group(const cqil_dims* dims, int P, const cqil_layer* layers, void* packed, size_t packed_bytes,
                    void* stream) {
    cqil_packed_layout L;
    int rc = packed_layout(dims, P, &L);
    if (rc) return rc;
    if (!layers || !packed) return CQIL_EINVAL;
    if (!aligned16(packed)) return CQIL_EINVAL;
    if (packed_bytes < L.total) return CQIL_ESIZE;
    PackArgs pa;
    for (int l = 0; l < P; ++l) {
        const cqil_layer& s = layers[l];
        const void* ptrs[9] = {s.wq, s.wk, s.wv, s.wo, s.wgate, s.wup, s.wdown, s.g_attn, s.g_ffn};
        for (const void* p : ptrs)
            if (!p || !aligned16(p)) return CQIL_EINVAL;
        pa.layers[l] = s;
    }
    hipError_t e = launch_pack(*dims, P, pa, (char*)packed, L, (hipStream_t)stream);
    return e == hipSuccess ? CQIL_OK : CQIL_EHIP;
}

static int group_forward_impl(const cqil_dims* dims, int P, int bypass_d, const void* packed, void* kc, void* vc,
                              int32_t* kv_len, int b_max, int max_kv_len, const void* x_in, void* x_out, int B, int T,
                              int advance, void* workspace, size_t workspace_bytes, hipStream_t st,
                              hipEvent_t* ev = nullptr, bool check_only = false, const void* x_res = nullptr) {
    StepArgs a;
    a.ev = ev;
    int rc = packed_layout(dims, P, &a.pl);
    if (rc) return rc;
    if (bypass_d < CQIL_ATTN_FFN_PARALLEL || B < 1 || T < 1) return CQIL_EINVAL;
    if (!packed || !kc || !vc || !kv_len || !x_in || !x_out || !workspace) return CQIL_EINVAL;
    if (!aligned16(packed) || !aligned16(kc) || !aligned16(vc) || !aligned16(x_in) || !aligned16(x_out) ||
        !aligned16(workspace) || !aligned16(x_res))
        return CQIL_EINVAL;
    if (b_max < 1 || max_kv_len < 0) return CQIL_EINVAL;
    if (B > b_max) return CQIL_ERANGE;
    if ((long long)max_kv_len + T > dims->max_seq) return CQIL_ERANGE;
    rc = ws_layout(dims, P, B, T, &a.wl);
    if (rc) return rc;
    if (workspace_bytes < a.wl.total) return CQIL_ESIZE;
    if (check_only) return CQIL_OK;
    a.d = *dims; a.P = P; a.bypass_d = bypass_d; a.B = B; a.T = T; a.advance = advance ? 1 : 0;
    a.packed = (const char*)packed;
    a.kc = kc; a.vc = vc; a.kv_len = kv_len; a.b_max = b_max; a.max_kv_len = max_kv_len;
    a.x_in = x_in; a.x_res = x_res ? x_res : x_in; a.x_out = x_out; a.ws = (char*)workspace;
    hipError_t e = (B * T == 1) ? launch_decode_step(a, st) : launch_generic_step(a, st);
    return e == hipSuccess ? CQIL_OK : CQIL_EHIP;
}

// chunks of tokens of the similarity kernels: enough workgroups to fill the chip, at least 4 tokens each
static void similarity_chunks(int L, int M, int* chunks, int* per) {
    const long pairs = (long)L * (L + 1) / 2;
    long c = (2048 + pairs - 1) / pairs;
    if (c > (M + 3) / 4) c = (M + 3) / 4;
    if (c < 1) c = 1;
    *per = (int)((M + c - 1) / c);
    *chunks = (M + *per - 1) / *per;
}

size_t cqil_input_similarity_workspace_bytes(int L, int M) {
    if (L < 1 || L > 1024 || M < 1) return 0;
    int chunks, per;
    similarity_chunks(L, M, &chunks, &per);
    return (size_t)chunks * L * L * sizeof(float);
}

int cqil_input_similarity(const void* X, int dtype, int L, int M, int n, float* sim, void* workspace,
                          size_t workspace_bytes, void* stream) {
    if (!X || !sim || !workspace) return CQIL_EINVAL;
    if (dtype != CQIL_F32 && dtype != CQIL_BF16) return CQIL_EINVAL;
    const int v = dtype == CQIL_BF16 ? 8 : 4;
    if (L < 1 || L > 1024 || M < 1 || n < v || n % v) return CQIL_EINVAL;
    if (!aligned16(X) || !aligned16(workspace)) return CQIL_EINVAL;
    if (workspace_bytes < cqil_input_similarity_workspace_bytes(L, M)) return CQIL_ESIZE;
    int chunks, per;
    similarity_chunks(L, M, &chunks, &per);
    return launch_similarity(X, dtype, L, M, n, sim, (float*)workspace, chunks, per, (hipStream_t)stream) == hipSuccess
               ? CQIL_OK
               : CQIL_EHIP;
}

int cqil_merge_lora(void* W, const void* A, const void* Bm, int dtype, int n_out, int n_in, int rank, float scale,
                    void* stream) {
    if (!W || !A || !Bm) return CQIL_EINVAL;
    if (dtype != CQIL_F32 && dtype != CQIL_BF16) return CQIL_EINVAL;
    const int v = dtype == CQIL_BF16 ? 8 : 4;
    if (n_out < 1 || n_in < v || n_in % v || rank < 1 || rank > 1024) return CQIL_EINVAL;
    if (!aligned16(W) || !aligned16(A)) return CQIL_EINVAL;
    return launch_merge_lora(W, A, Bm, dtype, n_out, n_in, rank, scale, (hipStream_t)stream) == hipSuccess ? CQIL_OK
                                                                                                             : CQIL_EHIP;
}

int cqil_group_forward(const cqil_dims* dims, int P, int bypass_d, const void* packed, cqil_kv* kv, const void* x_in,
                       void* x_out, int B, int T, int advance_kv_len, void* workspace, size_t workspace_bytes,
                       void* stream) {
    if (!kv) return CQIL_EINVAL;
    int rc = group_forward_impl(dims, P, bypass_d, packed, kv->k, kv->v, kv->kv_len, kv->b_max, kv->max_kv_len, x_in,
                                x_out, B, T, advance_kv_len, workspace, workspace_bytes, (hipStream_t)stream);
    if (rc == CQIL_OK && advance_kv_len) kv->max_kv_len += T;
    return rc;
}

int cqil_stream_read_probe(const void* buf, size_t bytes, void* sink, size_t sink_bytes, void* stream) {
    if (!buf || !sink || bytes < 16 || (bytes & 15)) return CQIL_EINVAL;
    if (!aligned16(buf) || ((uintptr_t)sink & 3)) return CQIL_EINVAL;
    if (sink_bytes < (size_t)kStreamProbeWorkgroups * sizeof(uint32_t)) return CQIL_ESIZE;
    return launch_stream_read(buf, bytes, (uint32_t*)sink, kStreamProbeWorkgroups, (hipStream_t)stream) == hipSuccess
               ? CQIL_OK
               : CQIL_EHIP;
}

size_t cqil_static_scratch_bytes(void) { return kStaticScratchBytes; }

int cqil_group_forward_static(const cqil_dims* dims, int P, int bypass_d, const void* packed, cqil_kv* kv,
                              const void* x_in, void* x_out, int B, int T, int advance_kv_len, void* stream) {
    if (!kv) return CQIL_EINVAL;
    WsLayout W;
    int rc = ws_layout(dims, P, B, T, &W);
    if (rc) return rc;
    if (W.total > kStaticScratchBytes) return CQIL_ESIZE;  // the step needs more scratch than the static array holds
    // every argument is checked before the first HIP call (a stand-in address takes the workspace's place)
    rc = group_forward_impl(dims, P, bypass_d, packed, kv->k, kv->v, kv->kv_len, kv->b_max, kv->max_kv_len, x_in, x_out,
                            B, T, advance_kv_len, (void*)kAlign, kStaticScratchBytes, (hipStream_t)stream, nullptr, true);
    if (rc) return rc;
    void* ws = nullptr;
    if ((rc = static_scratch(&ws)) != CQIL_OK) return rc;
    // nothing in the workspace has to start at zero: every kernel writes what a later one reads
    rc = group_forward_impl(dims, P, bypass_d, packed, kv->k, kv->v, kv->kv_len, kv->b_max, kv->max_kv_len, x_in, x_out,
                            B, T, advance_kv_len, ws, kStaticScratchBytes, (hipStream_t)stream);
    if (rc == CQIL_OK && advance_kv_len) kv->max_kv_len += T;
    return rc;
}

int cqil_decode_step_profile(const cqil_dims* dims, int P, int bypass_d, const void* packed, cqil_kv* kv,
                             const void* x_in, void* x_out, int B, void* workspace, size_t workspace_bytes,
                             void* stream, float* kernel_ms_out) {
    if (!kv || !kernel_ms_out) return CQIL_EINVAL;
    // only the single-token path (the six decode kernels) records events
    if (B != 1 || !dims) return CQIL_EINVAL;
    hipEvent_t ev[7];
    for (int i = 0; i < 7; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
            return CQIL_EHIP;
        }
    int rc = group_forward_impl(dims, P, bypass_d, packed, kv->k, kv->v, kv->kv_len, kv->b_max, kv->max_kv_len, x_in,
                                x_out, B, 1, 0, workspace, workspace_bytes, (hipStream_t)stream, ev);
    if (rc == CQIL_OK) {
        if (hipEventSynchronize(ev[6]) != hipSuccess) rc = CQIL_EHIP;
        for (int i = 0; i < 6 && rc == CQIL_OK; ++i)
            if (hipEventElapsedTime(&kernel_ms_out[i], ev[i], ev[i + 1]) != hipSuccess) rc = CQIL_EHIP;
    }
    for (int i = 0; i < 7; ++i) (void)hipEventDestroy(ev[i]);
    return rc;
}

// Model workspace: [hidden state (the groups update it in place)][logits][argmax scratch][group workspace]
static int model_ws(const cqil_model* m, int B, int T, size_t* x_off, size_t* logits_off, size_t* scratch_off,
                    size_t* group_off, size_t* total) {
    if (!m || !m->group_sizes || m->n_groups < 1 || m->vocab < 1 || B < 1 || T < 1) return CQIL_EINVAL;
    size_t gmax = 0;
    for (int g = 0; g < m->n_groups; ++g) {
        WsLayout W;
        int rc = ws_layout(&m->dims, m->group_sizes[g], B, T, &W);
        if (rc) return rc;
        if (W.total > gmax) gmax = W.total;
    }
    size_t off = 0;
    *x_off = off;       off = align_up(off + (size_t)B * T * m->dims.d_model * esize(m->dims.dtype));
    *logits_off = off;  off = align_up(off + (size_t)B * m->vocab * sizeof(float));
    *scratch_off = off; off = align_up(off + (size_t)B * 1024 * 2 * sizeof(float));
    *group_off = off;   off = align_up(off + gmax);
    *total = off;
    return CQIL_OK;
}

size_t cqil_model_workspace_bytes(const cqil_model* m, int B, int T) {
    size_t a, b, c, d, t;
    return model_ws(m, B, T, &a, &b, &c, &d, &t) ? 0 : t;
}

// Model loop shared by cqil_model_forward (sub_group < 0) and cqil_model_forward_substituted.
static int model_forward_impl(cqil_model* m, const int32_t* tokens, int B, int T, int bypass_d, int advance_kv_len,
                              int sub_group, int sub_k, void* hidden_out, float* logits_out, int32_t* next_token_out,
                              void* workspace, size_t workspace_bytes, void* stream) {
    size_t x_off, lg_off, sc_off, g_off, total;
    int rc = model_ws(m, B, T, &x_off, &lg_off, &sc_off, &g_off, &total);
    if (rc) return rc;
    if (!tokens || !workspace || !m->packed || !m->k_cache || !m->v_cache || !m->kv_len || !m->embedding ||
        !m->g_final || !m->lm_head)
        return CQIL_EINVAL;
    if (bypass_d < CQIL_ATTN_FFN_PARALLEL) return CQIL_EINVAL;
    if (!aligned16(workspace) || !aligned16(m->embedding) || !aligned16(m->lm_head) || !aligned16(m->g_final))
        return CQIL_EINVAL;
    if (hidden_out && !aligned16(hidden_out)) return CQIL_EINVAL;
    const bool subst = sub_group >= 0 && sub_k > 0;
    if (sub_group >= 0 && (sub_group >= m->n_groups || sub_k < 0 || sub_k > sub_group)) return CQIL_EINVAL;
    const size_t x_bytes = align_up((size_t)B * T * m->dims.d_model * esize(m->dims.dtype));
    if (workspace_bytes < total + (subst ? x_bytes : 0)) return CQIL_ESIZE;
    if (B > m->b_max) return CQIL_ERANGE;
    if ((long long)m->max_kv_len + T > m->dims.max_seq) return CQIL_ERANGE;
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;
    void* x = hidden_out ? hidden_out : (void*)(ws + x_off);
    void* x_sub = ws + total;   // the captured input of group sub_group - sub_k
    const size_t gbytes = total - g_off;
    // every group is checked (pointers, alignment, ranges, workspace) before the first launch
    for (int g = 0; g < m->n_groups; ++g) {
        rc = group_forward_impl(&m->dims, m->group_sizes[g], bypass_d, m->packed[g], m->k_cache[g], m->v_cache[g],
                                m->kv_len, m->b_max, m->max_kv_len, x, x, B, T, 0, ws + g_off, gbytes, st, nullptr, true);
        if (rc) return rc;
    }

    if (launch_embedding(m->dims, m->embedding, tokens, B * T, m->vocab, x, st) != hipSuccess) return CQIL_EHIP;
    for (int g = 0; g < m->n_groups; ++g) {
        if (subst && g == sub_group - sub_k &&
            launch_copy16(x, x_sub, (size_t)B * T * m->dims.d_model * esize(m->dims.dtype), st) != hipSuccess)
            return CQIL_EHIP;
        const bool here = subst && g == sub_group;
        // substituted group: its branches are computed from the captured state and added to the current one
        rc = group_forward_impl(&m->dims, m->group_sizes[g], bypass_d, m->packed[g], m->k_cache[g], m->v_cache[g],
                                m->kv_len, m->b_max, m->max_kv_len, here ? x_sub : x, x, B, T, 0, ws + g_off, gbytes, st,
                                nullptr, false, here ? x : nullptr);
        if (rc) return rc;
    }
    if (logits_out || next_token_out) {
        HeadArgs h;
        h.d = m->dims; h.vocab = m->vocab; h.B = B; h.T = T;
        h.hidden = x; h.g_final = m->g_final; h.lm_head = m->lm_head;
        h.logits = logits_out ? logits_out : (float*)(ws + lg_off);
        h.next_token = next_token_out;
        h.ws = ws + sc_off;
        if (launch_head(h, st) != hipSuccess) return CQIL_EHIP;
    }
    if (advance_kv_len) {
        if (launch_advance(m->kv_len, B, T, st) != hipSuccess) return CQIL_EHIP;
        m->max_kv_len += T;
    }
    return CQIL_OK;
}

int cqil_model_forward(cqil_model* m, const int32_t* tokens, int B, int T, int bypass_d, int advance_kv_len,
                       void* hidden_out, float* logits_out, int32_t* next_token_out, void* workspace,
                       size_t workspace_bytes, void* stream) {
    return model_forward_impl(m, tokens, B, T, bypass_d, advance_kv_len, -1, 0, hidden_out, logits_out, next_token_out,
                              workspace, workspace_bytes, stream);
}

size_t cqil_model_substituted_workspace_bytes(const cqil_model* m, int B, int T) {
    const size_t base = cqil_model_workspace_bytes(m, B, T);
    return base ? base + align_up((size_t)B * T * m->dims.d_model * esize(m->dims.dtype)) : 0;
}

int cqil_model_forward_substituted(cqil_model* m, const int32_t* tokens, int B, int T, int bypass_d, int advance_kv_len,
                                   int group, int k, void* hidden_out, float* logits_out, int32_t* next_token_out,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    if (group < 0) return CQIL_EINVAL;
    return model_forward_impl(m, tokens, B, T, bypass_d, advance_kv_len, group, k, hidden_out, logits_out,
                              next_token_out, workspace, workspace_bytes, stream);
}

}  // extern "C"
