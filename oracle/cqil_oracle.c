/*
 * CQIL oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of what the CQIL hot path computes
 * (Concurrent Computation of Quasi-Independent Layers, arxiv 2404.06709).  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may load this file.  It shares no
 * code, header, table or constant with the HIP path.
 *
 * Arithmetic: every activation, statistic and accumulation is IEEE double.  Weights are
 * read in their storage type (fp32, or bf16 bit patterns widened exactly) so that weight
 * quantisation is not counted as error.  No blocking, fusion or reordering beyond what the
 * equations state; OpenMP only splits independent output rows / heads between threads.
 *
 * What follows which passage of the paper:
 *   orc_attn_module   Eq.2: ATTN(x) = MHA(Norm(x)), heads, softmax(QK^T/sqrt(d_k))V, Concat(...)W^O
 *   orc_ffn_module    Eq.2: FFN(x) = W_2 f(W_1 Norm(x)), instantiated as LLaMA's bias-free SwiGLU
 *   orc_seq_layer     Eq.1: x_{l+1} = x_l + ATTN_l(x_l) + FFN_l(x_l + ATTN_l(x_l))
 *   orc_input_similarity   mean cosine similarity between the inputs of two layers (Sec.3.1)
 *   orc_merge_lora    W + BA, the merged form of the LoRA adapters the paper fine-tunes (Sec.5.1, App. C)
 *   orc_group_forward Eq.3 (d = 0) and Eq.4 (bypass distance d), Alg.1's middle loop
 *   orc_partition     Sec.4.2 "Layer Partition and Parallelism": (p, s, e) -> group sizes
 *   orc_model_forward Alg.1 as a whole, with the LLaMA embedding / final norm / lm head around it
 *   orc_model_forward_substituted   the input-substitution experiment of Sec.3.2 on that model
 *
 * Readings taken where the paper is silent or inconsistent (the same list is in the design
 * document): the bypass window is Eq.4's index set {l' : 1 <= l-l' <= d} (Alg.1's slice
 * expression is garbled); s..e are 1-indexed inclusive grouped layers (Sec.4.2's worked
 * example, not Alg.1's loop bounds); Norm = RMSNorm, f = SiLU gate, rotary embedding with
 * half-split pairing, causal mask and a per-layer KV cache are standard LLaMA-1, which the
 * paper uses but does not spell out.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };

typedef struct {
    int d_model, n_heads, head_dim, d_ffn, max_seq;
    double rope_base, rms_eps;
    int wdtype; /* storage type of every weight / gain / embedding pointer */
} orc_dims;

typedef struct {
    const void *wq, *wk, *wv, *wo;  /* [d_model, d_model], row-major [out, in] */
    const void *wgate, *wup;        /* [d_ffn, d_model] */
    const void *wdown;              /* [d_model, d_ffn] */
    const void *g_attn, *g_ffn;     /* [d_model] */
} orc_layer;

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* exact widening of one stored weight element to double */
static inline double wload(const void *w, int dtype, size_t i) {
    if (dtype == ORC_F32) return (double)((const float *)w)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)w)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* y[o] = sum_k W[o,k] x[k]  (the paper's xW with W stored [out,in]) */
void orc_linear(const void *W, int dtype, int n_out, int n_in, const double *x, double *y) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < n_out; ++o) {
        double acc = 0.0;
        size_t base = (size_t)o * (size_t)n_in;
        for (int k = 0; k < n_in; ++k) acc += wload(W, dtype, base + (size_t)k) * x[k];
        y[o] = acc;
    }
}

/* LoRA merge (Sec.5.1 / App. C: adapters on every linear matrix, alpha = rank, i.e. scale 1):
 *   out[o,k] = W[o,k] + scale * sum_j Bm[o,j] A[j,k]      W [n_out,n_in], A [r,n_in], Bm [n_out,r]
 * The sum is returned unrounded; the caller rounds it to the storage type. */
void orc_merge_lora(const void *W, const void *A, const void *Bm, int dtype, int n_out, int n_in, int r,
                    double scale, double *out) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < n_out; ++o)
        for (int k = 0; k < n_in; ++k) {
            double acc = 0.0;
            for (int j = 0; j < r; ++j)
                acc += wload(Bm, dtype, (size_t)o * (size_t)r + (size_t)j) * wload(A, dtype, (size_t)j * (size_t)n_in + (size_t)k);
            out[(size_t)o * (size_t)n_in + (size_t)k] = wload(W, dtype, (size_t)o * (size_t)n_in + (size_t)k) + scale * acc;
        }
}

/* Similarity of layer inputs (Sec.3.1): X [L][M][n] holds the inputs x_l of L layers for the same M tokens;
 *   sim[a][b] = (1/M) sum_m  <x_a[m], x_b[m]> / (|x_a[m]| |x_b[m]|)
 * (cosine per token, mean over tokens; a zero vector gives cosine 0). */
void orc_input_similarity(const double *X, int L, int M, int n, double *sim) {
    for (int a = 0; a < L; ++a)
        for (int b = 0; b < L; ++b) {
            double acc = 0.0;
            for (int m = 0; m < M; ++m) {
                const double *xa = X + ((size_t)a * (size_t)M + (size_t)m) * (size_t)n;
                const double *xb = X + ((size_t)b * (size_t)M + (size_t)m) * (size_t)n;
                double dot = 0.0, na = 0.0, nb = 0.0;
                for (int k = 0; k < n; ++k) { dot += xa[k] * xb[k]; na += xa[k] * xa[k]; nb += xb[k] * xb[k]; }
                if (na > 0.0 && nb > 0.0) acc += dot / (sqrt(na) * sqrt(nb));
            }
            sim[(size_t)a * (size_t)L + (size_t)b] = acc / (double)M;
        }
}

/* RMSNorm: out[k] = x[k] * g[k] / sqrt(mean_k x[k]^2 + eps) */
void orc_rmsnorm(const double *x, const void *g, int dtype, int n, double eps, double *out) {
    double ss = 0.0;
    for (int k = 0; k < n; ++k) ss += x[k] * x[k];
    double r = 1.0 / sqrt(ss / (double)n + eps);
    for (int k = 0; k < n; ++k) out[k] = x[k] * r * wload(g, dtype, (size_t)k);
}

/* Rotary embedding of one head vector at absolute position pos; pair (i, i + head_dim/2)
 * is rotated by the angle pos * base^(-2i/head_dim). */
void orc_rope(double *v, int head_dim, long pos, double base) {
    int half = head_dim / 2;
    for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)head_dim);
        double phi = (double)pos * theta;
        double c = cos(phi), s = sin(phi);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

double orc_silu(double z) { return z / (1.0 + exp(-z)); }

static size_t cache_index(const orc_dims *D, int b_max, int layer_in_group, int b, int h, long slot) {
    return ((((size_t)layer_in_group * (size_t)b_max + (size_t)b) * (size_t)D->n_heads + (size_t)h) *
                (size_t)D->max_seq + (size_t)slot) * (size_t)D->head_dim;
}

/*
 * ATTN_l(x) for one layer (Eq.2), for B sequences each bringing T new positions.
 *   x       [B][T][d_model]
 *   kcache, vcache: the group's caches [P][b_max][n_heads][max_seq][head_dim]; this layer is
 *                   index `lg` in them.  Slots kv_len[b] .. kv_len[b]+T-1 are written (K after
 *                   the rotary embedding), earlier slots are read.
 *   a_out   [B][T][d_model] = Concat(heads) W^O
 * Position t of sequence b attends slots 0 .. kv_len[b]+t (causal).
 * rows (may be NULL = every row): [B][T] flags.  A row whose flag is 0 still has its key and value computed
 * and cached (later rows attend them), but its query, attention and output are skipped and its a_out row is
 * left untouched: the outputs of the flagged rows are exactly those of the full call (Eq.2: an output row
 * depends on other rows only through their keys and values).  Used to sample rows of long prefills.
 */
static int attn_module_rows(const orc_dims *D, const orc_layer *L, int lg, double *kcache, double *vcache,
                            int b_max, const int32_t *kv_len, const double *x, int B, int T,
                            const unsigned char *rows, double *a_out) {
    const int dm = D->d_model, nh = D->n_heads, dk = D->head_dim;
    if (nh * dk != dm || (dk & 1)) return -1;
    double *nrm = malloc(sizeof(double) * (size_t)dm);
    double *q = malloc(sizeof(double) * (size_t)dm);
    double *k = malloc(sizeof(double) * (size_t)dm);
    double *v = malloc(sizeof(double) * (size_t)dm);
    double *ctx = malloc(sizeof(double) * (size_t)dm);
    if (!nrm || !q || !k || !v || !ctx) return -2;
    for (int b = 0; b < B; ++b) {
        if (kv_len[b] < 0 || kv_len[b] + T > D->max_seq) return -3;
        for (int t = 0; t < T; ++t) {
            const double *xt = x + ((size_t)b * (size_t)T + (size_t)t) * (size_t)dm;
            long pos = (long)kv_len[b] + t;
            const int want = !rows || rows[(size_t)b * (size_t)T + (size_t)t];
            orc_rmsnorm(xt, L->g_attn, D->wdtype, dm, D->rms_eps, nrm);
            if (want) orc_linear(L->wq, D->wdtype, dm, dm, nrm, q);
            orc_linear(L->wk, D->wdtype, dm, dm, nrm, k);
            orc_linear(L->wv, D->wdtype, dm, dm, nrm, v);
#pragma omp parallel for schedule(static)
            for (int h = 0; h < nh; ++h) {
                double *qh = q + (size_t)h * dk, *kh = k + (size_t)h * dk, *vh = v + (size_t)h * dk;
                orc_rope(kh, dk, pos, D->rope_base);
                memcpy(kcache + cache_index(D, b_max, lg, b, h, pos), kh, sizeof(double) * (size_t)dk);
                memcpy(vcache + cache_index(D, b_max, lg, b, h, pos), vh, sizeof(double) * (size_t)dk);
                if (!want) continue;
                orc_rope(qh, dk, pos, D->rope_base);
                /* softmax(q K^T / sqrt(d_k)) V over slots 0..pos */
                double *sc = malloc(sizeof(double) * (size_t)(pos + 1));
                double mx = -INFINITY;
                for (long j = 0; j <= pos; ++j) {
                    const double *kj = kcache + cache_index(D, b_max, lg, b, h, j);
                    double s = 0.0;
                    for (int e = 0; e < dk; ++e) s += qh[e] * kj[e];
                    s /= sqrt((double)dk);
                    sc[j] = s;
                    if (s > mx) mx = s;
                }
                double den = 0.0;
                for (long j = 0; j <= pos; ++j) { sc[j] = exp(sc[j] - mx); den += sc[j]; }
                double *ch = ctx + (size_t)h * dk;
                for (int e = 0; e < dk; ++e) ch[e] = 0.0;
                for (long j = 0; j <= pos; ++j) {
                    const double *vj = vcache + cache_index(D, b_max, lg, b, h, j);
                    double p = sc[j] / den;
                    for (int e = 0; e < dk; ++e) ch[e] += p * vj[e];
                }
                free(sc);
            }
            if (want)
                orc_linear(L->wo, D->wdtype, dm, dm, ctx,
                           a_out + ((size_t)b * (size_t)T + (size_t)t) * (size_t)dm);
        }
    }
    free(nrm); free(q); free(k); free(v); free(ctx);
    return 0;
}

int orc_attn_module(const orc_dims *D, const orc_layer *L, int lg, double *kcache, double *vcache,
                    int b_max, const int32_t *kv_len, const double *x, int B, int T, double *a_out) {
    return attn_module_rows(D, L, lg, kcache, vcache, b_max, kv_len, x, B, T, NULL, a_out);
}

/* FFN_l(h) for M token vectors (Eq.2 with SwiGLU): Wdown( silu(Wgate n) * (Wup n) ), n = Norm(h) */
int orc_ffn_module(const orc_dims *D, const orc_layer *L, const double *h, int M, double *out) {
    const int dm = D->d_model, f = D->d_ffn;
    double *nrm = malloc(sizeof(double) * (size_t)dm);
    double *g = malloc(sizeof(double) * (size_t)f);
    double *u = malloc(sizeof(double) * (size_t)f);
    if (!nrm || !g || !u) return -2;
    for (int m = 0; m < M; ++m) {
        orc_rmsnorm(h + (size_t)m * dm, L->g_ffn, D->wdtype, dm, D->rms_eps, nrm);
        orc_linear(L->wgate, D->wdtype, f, dm, nrm, g);
        orc_linear(L->wup, D->wdtype, f, dm, nrm, u);
        for (int j = 0; j < f; ++j) u[j] = orc_silu(g[j]) * u[j];
        orc_linear(L->wdown, D->wdtype, dm, f, u, out + (size_t)m * dm);
    }
    free(nrm); free(g); free(u);
    return 0;
}

/* Eq.1: one ordinary pre-norm decoder layer.  Cache arrays are [1][b_max][n][max_seq][d_k]. */
int orc_seq_layer(const orc_dims *D, const orc_layer *L, double *kcache, double *vcache, int b_max,
                  const int32_t *kv_len, const double *x, double *x_out, int B, int T) {
    size_t n = (size_t)B * (size_t)T * (size_t)D->d_model;
    double *a = malloc(sizeof(double) * n), *fo = malloc(sizeof(double) * n);
    if (!a || !fo) return -2;
    int rc = orc_attn_module(D, L, 0, kcache, vcache, b_max, kv_len, x, B, T, a);
    if (rc) return rc;
    for (size_t i = 0; i < n; ++i) a[i] = x[i] + a[i]; /* a_l = x_l + ATTN_l(x_l) */
    rc = orc_ffn_module(D, L, a, B * T, fo);
    if (rc) return rc;
    for (size_t i = 0; i < n; ++i) x_out[i] = a[i] + fo[i];
    free(a); free(fo);
    return 0;
}

/*
 * Eq.4 (Eq.3 when d = 0): P layers read the same x.
 *   attn_i = ATTN_{l_i}(x)                                      i = 0..P-1, each with its own cache
 *   h_i    = x + attn_i + sum_{j : 1 <= i-j <= d} attn_j         FFN input of layer i (bypass)
 *   x_out  = x + sum_i attn_i + sum_i FFN_{l_i}(h_i)
 * d = -1 selects the attention-FFN parallel form of App. A (Eq.5), applied to every layer of the group:
 *   h_i    = x                                                   (the feed-forward module reads the shared input)
 *   x_out  = x + sum_i attn_i + sum_i FFN_{l_i}(x)
 * dbg_attn, dbg_h: optional [P][B][T][d_model] copies of attn_i and h_i (may be NULL).
 * kv_len is not advanced here.
 */
static int group_forward_rows(const orc_dims *D, int P, int d, const orc_layer *layers, double *kcache,
                              double *vcache, int b_max, const int32_t *kv_len, const double *x, double *x_out,
                              int B, int T, const unsigned char *rows, double *dbg_attn, double *dbg_h);

int orc_group_forward(const orc_dims *D, int P, int d, const orc_layer *layers, double *kcache,
                      double *vcache, int b_max, const int32_t *kv_len, const double *x, double *x_out,
                      int B, int T, double *dbg_attn, double *dbg_h) {
    return group_forward_rows(D, P, d, layers, kcache, vcache, b_max, kv_len, x, x_out, B, T, NULL, dbg_attn, dbg_h);
}

/* The same step with the outputs restricted to the rows whose flag in rows[B][T] is non-zero: every row's keys and
 * values are computed and cached, the flagged rows of x_out / dbg_attn / dbg_h are exactly those of the full call,
 * the other rows of the outputs are zero.  The feed-forward module acts on each row alone (Eq.2), so skipping a
 * row changes no other row. */
int orc_group_forward_rows(const orc_dims *D, int P, int d, const orc_layer *layers, double *kcache,
                           double *vcache, int b_max, const int32_t *kv_len, const double *x, double *x_out,
                           int B, int T, const unsigned char *rows, double *dbg_attn, double *dbg_h) {
    if (!rows) return -1;
    return group_forward_rows(D, P, d, layers, kcache, vcache, b_max, kv_len, x, x_out, B, T, rows, dbg_attn, dbg_h);
}

static int group_forward_rows(const orc_dims *D, int P, int d, const orc_layer *layers, double *kcache,
                              double *vcache, int b_max, const int32_t *kv_len, const double *x, double *x_out,
                              int B, int T, const unsigned char *rows, double *dbg_attn, double *dbg_h) {
    if (P < 1 || d < -1) return -1;
    size_t n = (size_t)B * (size_t)T * (size_t)D->d_model;
    double *attn = calloc(n * (size_t)P, sizeof(double));
    double *h = malloc(sizeof(double) * n);
    double *fo = calloc(n, sizeof(double));
    double *acc = malloc(sizeof(double) * n);
    if (!attn || !h || !fo || !acc) return -2;
    for (int i = 0; i < P; ++i) {
        int rc = attn_module_rows(D, &layers[i], i, kcache, vcache, b_max, kv_len, x, B, T, rows, attn + n * (size_t)i);
        if (rc) return rc;
    }
    memcpy(acc, x, sizeof(double) * n);
    for (int i = 0; i < P; ++i)
        for (size_t e = 0; e < n; ++e) acc[e] += attn[n * (size_t)i + e];
    for (int i = 0; i < P; ++i) {
        if (d == -1) {
            memcpy(h, x, sizeof(double) * n);                              /* Eq.5 */
        } else {
            for (size_t e = 0; e < n; ++e) h[e] = x[e] + attn[n * (size_t)i + e];
        }
        for (int j = 0; j < P; ++j) {
            int dist = i - j;
            if (dist >= 1 && dist <= d)
                for (size_t e = 0; e < n; ++e) h[e] += attn[n * (size_t)j + e];
        }
        if (dbg_h) memcpy(dbg_h + n * (size_t)i, h, sizeof(double) * n);
        if (!rows) {
            int rc = orc_ffn_module(D, &layers[i], h, B * T, fo);
            if (rc) return rc;
        } else {
            for (int m = 0; m < B * T; ++m) {   /* row by row: the module treats every row alone */
                if (!rows[m]) continue;
                int rc = orc_ffn_module(D, &layers[i], h + (size_t)m * D->d_model, 1, fo + (size_t)m * D->d_model);
                if (rc) return rc;
            }
        }
        for (size_t e = 0; e < n; ++e) acc[e] += fo[e];
    }
    if (rows)   /* rows that were not asked for are reported as zero, not as partial sums */
        for (int m = 0; m < B * T; ++m)
            if (!rows[m]) {
                memset(acc + (size_t)m * D->d_model, 0, sizeof(double) * (size_t)D->d_model);
                if (dbg_h) for (int i = 0; i < P; ++i) memset(dbg_h + n * (size_t)i + (size_t)m * D->d_model, 0, sizeof(double) * (size_t)D->d_model);
            }
    if (dbg_attn) memcpy(dbg_attn, attn, sizeof(double) * n * (size_t)P);
    memcpy(x_out, acc, sizeof(double) * n);
    free(attn); free(h); free(fo); free(acc);
    return 0;
}

/* number of (source, destination) bypass transfers inside one group of p layers */
int orc_bypass_transfers(int p, int d) {
    int cnt = 0;
    for (int i = 0; i < p; ++i)
        for (int j = 0; j < p; ++j)
            if (i - j >= 1 && i - j <= d) ++cnt;
    return cnt;
}

/* Sec.4.2: layers s..e (1-indexed, inclusive) go into consecutive groups of at most p, every
 * other layer is a group of one.  Returns the number of groups, sizes in group_sizes[<= L]. */
int orc_partition(int L, int p, int s, int e, int *group_sizes) {
    if (L < 1 || p < 1 || s < 1 || e > L || s > e + 1) return -1;
    int n = 0, l = 1;
    while (l <= L) {
        if (l >= s && l <= e) {
            int left = e - l + 1;
            int sz = left < p ? left : p;
            group_sizes[n++] = sz;
            l += sz;
        } else {
            group_sizes[n++] = 1;
            l += 1;
        }
    }
    return n;
}

/*
 * Whole model: x_1 = embedding[token]; groups in layer order; final RMSNorm; logits = W_lm n;
 * greedy next token = lowest index among the maxima.
 *   layers       [L] in model order; group_sizes [n_groups] sums to L
 *   kcache/vcache [L][b_max][n][max_seq][d_k] (layer-major, so a group's caches are contiguous)
 *   hidden_out   optional [B][T][d_model] final hidden state (before the final norm)
 *   logits_out   optional [B][vocab] for the last new position
 *   next_out     optional [B]
 * kv_len is not advanced here.
 */
static int model_forward_subst(const orc_dims *D, int L, const orc_layer *layers, int n_groups,
                               const int *group_sizes, int d, int sub_group, int sub_k, const void *embedding,
                               const void *g_final, const void *lm_head, int vocab, double *kcache, double *vcache,
                               int b_max, const int32_t *kv_len, const int32_t *tokens, int B, int T,
                               double *hidden_out, double *logits_out, int32_t *next_out);

int orc_model_forward(const orc_dims *D, int L, const orc_layer *layers, int n_groups,
                      const int *group_sizes, int d, const void *embedding, const void *g_final,
                      const void *lm_head, int vocab, double *kcache, double *vcache, int b_max,
                      const int32_t *kv_len, const int32_t *tokens, int B, int T, double *hidden_out,
                      double *logits_out, int32_t *next_out) {
    return model_forward_subst(D, L, layers, n_groups, group_sizes, d, -1, 0, embedding, g_final, lm_head, vocab, kcache,
                               vcache, b_max, kv_len, tokens, B, T, hidden_out, logits_out, next_out);
}

/*
 * Input substitution (Sec.3.2): with the model written as x_{L+1} = x_1 + F_1(x_1) + ... + F_L(x_L), the input of
 * one F is replaced by the input of an earlier one and every other term is kept: here F is the update of group
 * sub_group (a layer when every group has one layer) and it reads the input of group sub_group - sub_k,
 *   x_after = x_before + ( group_forward(x_input_of(sub_group - sub_k)) - x_input_of(sub_group - sub_k) ),
 * later groups see the changed state; the group's caches are filled from the substituted input.
 * sub_k = 0 is the plain model.  Requires 0 <= sub_k <= sub_group < n_groups.
 */
int orc_model_forward_substituted(const orc_dims *D, int L, const orc_layer *layers, int n_groups,
                                  const int *group_sizes, int d, int sub_group, int sub_k, const void *embedding,
                                  const void *g_final, const void *lm_head, int vocab, double *kcache, double *vcache,
                                  int b_max, const int32_t *kv_len, const int32_t *tokens, int B, int T,
                                  double *hidden_out, double *logits_out, int32_t *next_out) {
    if (sub_group < 0 || sub_group >= n_groups || sub_k < 0 || sub_k > sub_group) return -1;
    return model_forward_subst(D, L, layers, n_groups, group_sizes, d, sub_group, sub_k, embedding, g_final, lm_head,
                               vocab, kcache, vcache, b_max, kv_len, tokens, B, T, hidden_out, logits_out, next_out);
}

static int model_forward_subst(const orc_dims *D, int L, const orc_layer *layers, int n_groups,
                               const int *group_sizes, int d, int sub_group, int sub_k, const void *embedding,
                               const void *g_final, const void *lm_head, int vocab, double *kcache, double *vcache,
                               int b_max, const int32_t *kv_len, const int32_t *tokens, int B, int T,
                               double *hidden_out, double *logits_out, int32_t *next_out) {
    const int dm = D->d_model;
    size_t n = (size_t)B * (size_t)T * (size_t)dm;
    double *x = malloc(sizeof(double) * n), *y = malloc(sizeof(double) * n);
    double *xs = malloc(sizeof(double) * n); /* input of group sub_group - sub_k */
    if (!x || !y || !xs) return -2;
    for (int m = 0; m < B * T; ++m) {
        int32_t tok = tokens[m];
        if (tok < 0 || tok >= vocab) return -4;
        for (int k = 0; k < dm; ++k) x[(size_t)m * dm + k] = wload(embedding, D->wdtype, (size_t)tok * dm + k);
    }
    size_t per_layer = (size_t)b_max * (size_t)D->n_heads * (size_t)D->max_seq * (size_t)D->head_dim;
    int l0 = 0;
    for (int g = 0; g < n_groups; ++g) {
        int P = group_sizes[g];
        if (P < 1 || l0 + P > L) return -1;
        const int subst = sub_group >= 0 && sub_k > 0;
        if (subst && g == sub_group - sub_k) memcpy(xs, x, sizeof(double) * n);
        const double *in = (subst && g == sub_group) ? xs : x;
        int rc = orc_group_forward(D, P, d, layers + l0, kcache + per_layer * (size_t)l0,
                                   vcache + per_layer * (size_t)l0, b_max, kv_len, in, y, B, T, NULL, NULL);
        if (rc) return rc;
        if (subst && g == sub_group)   /* the group's update F(xs) = y - xs, added to the current state */
            for (size_t e = 0; e < n; ++e) y[e] = x[e] + (y[e] - xs[e]);
        double *tmp = x; x = y; y = tmp;
        l0 += P;
    }
    if (l0 != L) return -1;
    if (hidden_out) memcpy(hidden_out, x, sizeof(double) * n);
    if (logits_out || next_out) {
        double *nrm = malloc(sizeof(double) * (size_t)dm);
        double *lg = malloc(sizeof(double) * (size_t)vocab);
        if (!nrm || !lg) return -2;
        for (int b = 0; b < B; ++b) {
            const double *xl = x + ((size_t)b * T + (size_t)(T - 1)) * dm;
            orc_rmsnorm(xl, g_final, D->wdtype, dm, D->rms_eps, nrm);
            orc_linear(lm_head, D->wdtype, vocab, dm, nrm, lg);
            if (logits_out) memcpy(logits_out + (size_t)b * vocab, lg, sizeof(double) * (size_t)vocab);
            if (next_out) {
                int best = 0;
                for (int j = 1; j < vocab; ++j)
                    if (lg[j] > lg[best]) best = j;
                next_out[b] = best;
            }
        }
        free(nrm); free(lg);
    }
    free(x); free(y); free(xs);
    return 0;
}
