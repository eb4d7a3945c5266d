/*
 * CPU oracle (see ee_oracle.h).  TEST INFRASTRUCTURE ONLY.
 *
 * Plain loops in the paper's order: embedding -> for each layer the
 * pre-norm attention block and the pre-norm SwiGLU block (Eq. 3, the layer
 * recurrence h^(l) = f^(l)(h^(l-1)); f is the Llama-2 block of the models the
 * paper evaluates) -> LM head on the hidden state of the requested layers
 * (z^(l) = LMHead(h^(l))) -> greedy accept rule (Eq. 2 / Eq. 5).
 *
 * No blocking, fusion or reordering; OpenMP only spreads independent output
 * elements over threads, and "omp simd" lets the compiler vectorise the dot
 * product's sum.
 */
#include "ee_oracle.h"

#include <fcntl.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <unistd.h>

#ifndef EO_REAL
#define EO_REAL float
#endif
typedef EO_REAL real;

#define HEADER_BYTES 256
#define ALIGN_BYTES 256

typedef struct {
    const uint16_t *g_attn, *wq, *wk, *wv, *wo, *g_ffn, *wg, *wu, *wd;
} layer_w;

struct eo_model {
    eo_config c;
    void *map;
    size_t map_bytes;
    const uint16_t *emb, *g_final, *w_lm;
    const uint16_t *g_exit[EO_MAX_EXITS];
    /* exit-head adapters (n_ad bottlenecks of width ad_w each, A = n_ad * ad_w), per stored exit */
    int n_ad, ad_w;
    const uint16_t *ad_down[EO_MAX_EXITS];  /* [A][d]    */
    const uint16_t *ad_bdown[EO_MAX_EXITS]; /* [A]       */
    const uint16_t *ad_up[EO_MAX_EXITS];    /* [d][A]    */
    const uint16_t *ad_bup[EO_MAX_EXITS];   /* [n_ad][d] */
    layer_w *layers;
};

struct eo_session {
    const eo_model *m;
    int max_ctx;
    int kv_len;
    int has_pending;
    int32_t pending;
    int last_P, last_M; /* position and rows of the last verify pass (for eo_commit_rows) */
    real *kc; /* [L][max_ctx][d] */
    real *vc; /* [L][max_ctx][d] */
};

int eo_sizeof_real(void) { return (int)sizeof(real); }

/* ---------- leaf arithmetic ---------- */

static inline real bf16_val(uint16_t b)
{
    union { uint32_t u; float f; } v;
    v.u = ((uint32_t)b) << 16;
    return (real)v.f;
}

/* sum_k w[k] * x[k] */
static inline real dot_w(const uint16_t *w, const real *x, int n)
{
    real s = 0;
#pragma omp simd reduction(+ : s)
    for (int k = 0; k < n; ++k)
        s += bf16_val(w[k]) * x[k];
    return s;
}

static inline real dot_rr(const real *a, const real *b, int n)
{
    real s = 0;
#pragma omp simd reduction(+ : s)
    for (int k = 0; k < n; ++k)
        s += a[k] * b[k];
    return s;
}

/* y[m][n] = sum_k W[n][k] x[m][k]   (W is [N][K] row-major).
   target_clones only selects the widest vector unit of the host at load time;
   the loop is the same in every clone. */
__attribute__((target_clones("avx512f", "avx2", "default")))
static void linear(const uint16_t *W, int N, int K, const real *x, int M, real *y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m)
            y[(size_t)m * N + n] = dot_w(W + (size_t)n * K, x + (size_t)m * K, K);
}

/* out = x / sqrt(mean(x^2) + eps) * g, row by row */
static void rmsnorm(const real *x, const uint16_t *g, int M, int d, real eps, real *out)
{
    for (int m = 0; m < M; ++m) {
        const real *xr = x + (size_t)m * d;
        real ss = 0;
        for (int k = 0; k < d; ++k)
            ss += xr[k] * xr[k];
        real inv = (real)1 / (real)sqrt((double)(ss / (real)d + eps));
        for (int k = 0; k < d; ++k)
            out[(size_t)m * d + k] = xr[k] * inv * bf16_val(g[k]);
    }
}

/* Rotary embedding, half-split pairing (i, i + hd/2) inside each head:
   theta_i = base^(-2i/hd), angle = pos * theta_i. */
static void rope_row(real *x, int n_heads, int hd, int pos, double base)
{
    int half = hd / 2;
    for (int h = 0; h < n_heads; ++h) {
        real *p = x + (size_t)h * hd;
        for (int i = 0; i < half; ++i) {
            double theta = pow(base, -2.0 * (double)i / (double)hd);
            double ang = (double)pos * theta;
            real c = (real)cos(ang), s = (real)sin(ang);
            real a = p[i], b = p[i + half];
            p[i] = a * c - b * s;
            p[i + half] = b * c + a * s;
        }
    }
}

static inline real silu(real x) { return x / ((real)1 + (real)exp(-(double)x)); }

/* softmax(scores[0..n)) in place, subtracting the maximum */
static void softmax_inplace(real *s, int n)
{
    real mx = s[0];
    for (int i = 1; i < n; ++i)
        if (s[i] > mx) mx = s[i];
    real sum = 0;
    for (int i = 0; i < n; ++i) {
        s[i] = (real)exp((double)(s[i] - mx));
        sum += s[i];
    }
    for (int i = 0; i < n; ++i)
        s[i] /= sum;
}

static int argmax_lowest(const real *z, int n)
{
    int best = 0;
    for (int i = 1; i < n; ++i)
        if (z[i] > z[best]) best = i;
    return best;
}

/* Confidence score of one row (paper Eq. 4): the largest entry of softmax(z), the definition
   written out: p_j = exp(z_j - max z) / sum_i exp(z_i - max z), then the maximum of p. */
static double max_softmax(const real *z, int n)
{
    real mx = z[0];
    for (int i = 1; i < n; ++i)
        if (z[i] > mx) mx = z[i];
    real sum = 0;
    for (int i = 0; i < n; ++i)
        sum += (real)exp((double)(z[i] - mx));
    real best = 0;
    for (int i = 0; i < n; ++i) {
        real p = (real)exp((double)(z[i] - mx)) / sum;
        if (p > best) best = p;
    }
    return (double)best;
}

/* Accept rule (Eq. 2): delta = longest prefix with drafts[j] == a[j]; next = a[delta] */
static void accept_rule(const int32_t *drafts, int gamma, const int32_t *a, int32_t *delta,
                        int32_t *next)
{
    int d = 0;
    while (d < gamma && drafts[d] == a[d])
        ++d;
    *delta = d;
    if (next) *next = a[d];
}

/* ---------- model file ---------- */

static size_t align_up(size_t x) { return (x + ALIGN_BYTES - 1) / ALIGN_BYTES * ALIGN_BYTES; }

static const uint16_t *take(const uint8_t *base, size_t *off, size_t n_elems)
{
    *off = align_up(*off);
    const uint16_t *p = (const uint16_t *)(base + *off);
    *off += 2 * n_elems;
    return p;
}

int eo_model_open(const char *path, eo_model **out)
{
    int fd = open(path, O_RDONLY);
    if (fd < 0) return EO_EIO;
    struct stat st;
    if (fstat(fd, &st) != 0) { close(fd); return EO_EIO; }
    if ((size_t)st.st_size < HEADER_BYTES) { close(fd); return EO_EFORMAT; }
    void *map = mmap(NULL, (size_t)st.st_size, PROT_READ, MAP_SHARED, fd, 0);
    close(fd);
    if (map == MAP_FAILED) return EO_EIO;
    const uint8_t *b = (const uint8_t *)map;
    if (memcmp(b, "EEVMODL1", 8) != 0) { munmap(map, (size_t)st.st_size); return EO_EFORMAT; }
    uint32_t u[8];
    memcpy(u, b + 8, sizeof u);
    eo_model *m = (eo_model *)calloc(1, sizeof *m);
    m->map = map;
    m->map_bytes = (size_t)st.st_size;
    if (u[0] != 1) { eo_model_close(m); return EO_EFORMAT; }
    m->c.n_layers = (int32_t)u[1];
    m->c.d_model = (int32_t)u[2];
    m->c.n_heads = (int32_t)u[3];
    m->c.head_dim = (int32_t)u[4];
    m->c.d_ffn = (int32_t)u[5];
    m->c.vocab = (int32_t)u[6];
    m->c.n_exits = (int32_t)u[7];
    memcpy(&m->c.rope_base, b + 40, 4);
    memcpy(&m->c.rms_eps, b + 44, 4);
    if (m->c.n_exits < 0 || m->c.n_exits > EO_MAX_EXITS || m->c.n_layers < 1 ||
        m->c.n_heads * m->c.head_dim != m->c.d_model || (m->c.head_dim & 1)) {
        eo_model_close(m);
        return EO_EFORMAT;
    }
    uint32_t ex[EO_MAX_EXITS];
    memcpy(ex, b + 48, sizeof ex);
    for (int i = 0; i < m->c.n_exits; ++i)
        m->c.exit_layers[i] = (int32_t)ex[i];

    size_t d = (size_t)m->c.d_model, F = (size_t)m->c.d_ffn, V = (size_t)m->c.vocab;
    size_t off = HEADER_BYTES;
    m->emb = take(b, &off, V * d);
    m->layers = (layer_w *)calloc((size_t)m->c.n_layers, sizeof(layer_w));
    for (int l = 0; l < m->c.n_layers; ++l) {
        layer_w *w = &m->layers[l];
        w->g_attn = take(b, &off, d);
        w->wq = take(b, &off, d * d);
        w->wk = take(b, &off, d * d);
        w->wv = take(b, &off, d * d);
        w->wo = take(b, &off, d * d);
        w->g_ffn = take(b, &off, d);
        w->wg = take(b, &off, F * d);
        w->wu = take(b, &off, F * d);
        w->wd = take(b, &off, d * F);
    }
    m->g_final = take(b, &off, d);
    m->w_lm = take(b, &off, V * d);
    for (int i = 0; i < m->c.n_exits; ++i)
        m->g_exit[i] = take(b, &off, d);
    {
        uint32_t ad[2];
        memcpy(ad, b + 208, sizeof ad);
        m->n_ad = (int)ad[0];
        m->ad_w = (int)ad[1];
        if ((m->n_ad == 0) != (m->ad_w == 0) || m->n_ad < 0 || m->n_ad > 64 || m->ad_w < 0 || m->ad_w > 65536) {
            eo_model_close(m);
            return EO_EFORMAT;
        }
        const size_t A = (size_t)m->n_ad * (size_t)m->ad_w;
        for (int i = 0; A && i < m->c.n_exits; ++i) {
            m->ad_down[i] = take(b, &off, A * d);
            m->ad_bdown[i] = take(b, &off, A);
            m->ad_up[i] = take(b, &off, d * A);
            m->ad_bup[i] = take(b, &off, (size_t)m->n_ad * d);
        }
    }
    if (align_up(off) > m->map_bytes) { eo_model_close(m); return EO_EFORMAT; }
    *out = m;
    return EO_OK;
}

void eo_model_close(eo_model *m)
{
    if (!m) return;
    if (m->map) munmap(m->map, m->map_bytes);
    free(m->layers);
    free(m);
}

int eo_model_config(const eo_model *m, eo_config *out)
{
    if (!m || !out) return EO_EINVAL;
    *out = m->c;
    return EO_OK;
}

/* index of the stored exit head after layer e, or -1 */
static int exit_slot(const eo_model *m, int e)
{
    for (int i = 0; i < m->c.n_exits; ++i)
        if (m->c.exit_layers[i] == e) return i;
    return -1;
}

/* gain vector of the exit head after layer e, or NULL */
static const uint16_t *exit_gain(const eo_model *m, int e)
{
    for (int i = 0; i < m->c.n_exits; ++i)
        if (m->c.exit_layers[i] == e) return m->g_exit[i];
    return NULL;
}

/* ---------- sessions ---------- */

int eo_session_new(const eo_model *m, int max_ctx, eo_session **out)
{
    if (!m || max_ctx < 1 || !out) return EO_EINVAL;
    eo_session *s = (eo_session *)calloc(1, sizeof *s);
    s->m = m;
    s->max_ctx = max_ctx;
    size_t n = (size_t)m->c.n_layers * (size_t)max_ctx * (size_t)m->c.d_model;
    s->kc = (real *)calloc(n, sizeof(real));
    s->vc = (real *)calloc(n, sizeof(real));
    if (!s->kc || !s->vc) { eo_session_free(s); return EO_ECAPACITY; }
    *out = s;
    return EO_OK;
}

void eo_session_free(eo_session *s)
{
    if (!s) return;
    free(s->kc);
    free(s->vc);
    free(s);
}

int eo_kv_len(const eo_session *s) { return s ? s->kv_len : EO_EINVAL; }

int eo_pending(const eo_session *s, int32_t *token)
{
    if (!s || !s->has_pending) return EO_ESTATE;
    *token = s->pending;
    return EO_OK;
}

int eo_set_pending(eo_session *s, int32_t token)
{
    if (!s || token < 0 || token >= s->m->c.vocab) return EO_EINVAL;
    s->pending = token;
    s->has_pending = 1;
    return EO_OK;
}

int eo_kv_truncate(eo_session *s, int new_len)
{
    if (!s || new_len < 0 || new_len > s->kv_len) return EO_EINVAL;
    s->kv_len = new_len; /* entries past new_len are stale and get overwritten */
    return EO_OK;
}

/* Commit of a verify pass whose accept decision was taken outside (probabilistic verification,
   Eq. 2 with the draft probabilities): the first delta+1 rows of the last pass become part of
   the sequence (their K/V are in the cache already) and `token` becomes the pending token. */
int eo_commit_rows(eo_session *s, int delta, int32_t token)
{
    if (!s || s->last_M < 1 || delta < 0 || delta >= s->last_M) return EO_EINVAL;
    if (token < 0 || token >= s->m->c.vocab) return EO_EINVAL;
    s->kv_len = s->last_P + delta + 1;
    s->pending = token;
    s->has_pending = 1;
    return EO_OK;
}

/* ---------- exit head with adapters ---------- */

/* The paper's exit heads are "adapter layers after each layer" that connect the layer's
   output to the shared LM head (Methodology, early-exit fine-tuning; Experimental Setup);
   the trainable-parameter counts of its fine-tuning table equal three bias-carrying
   bottlenecks of width 128 per layer.  Reading taken here: the n_ad bottlenecks act in
   parallel on the layer's output and their results are added to it,
       a = h + sum_j ( W_up,j . silu(W_down,j . h + b_down,j) + b_up,j ),
   and the exit's logits are LMHead(RMSNorm(a; g_exit)).  The bottlenecks' rows are stored
   one after the other (W_down [A][d], W_up [d][A], A = n_ad * width), so the sum over j is the
   sum over all A hidden units.  h: [M][d] (left unchanged), a: [M][d]. */
static void adapter_rows(const eo_model *m, int slot, const real *h, int M, real *a)
{
    const int d = m->c.d_model, A = m->n_ad * m->ad_w;
    real *t = (real *)malloc((size_t)M * A * sizeof(real));
    linear(m->ad_down[slot], A, d, h, M, t);
    for (int i = 0; i < M; ++i)
        for (int r = 0; r < A; ++r)
            t[(size_t)i * A + r] = silu(t[(size_t)i * A + r] + bf16_val(m->ad_bdown[slot][r]));
    linear(m->ad_up[slot], d, A, t, M, a);
    for (int i = 0; i < M; ++i)
        for (int c = 0; c < d; ++c) {
            real b = 0;
            for (int j = 0; j < m->n_ad; ++j)
                b += bf16_val(m->ad_bup[slot][(size_t)j * d + c]);
            a[(size_t)i * d + c] = h[(size_t)i * d + c] + a[(size_t)i * d + c] + b;
        }
    free(t);
}

/* ---------- one pass over M rows with the KV cache ---------- */

typedef struct {
    int n_heads;                       /* number of LM-head evaluations requested        */
    int layer[EO_MAX_EXITS + 1];       /* after which layer (L for the final head)        */
    const uint16_t *gain[EO_MAX_EXITS + 1];
    real *logits[EO_MAX_EXITS + 1];    /* each [M][V]                                     */
} head_req;

static void copy_trace(double *dst, const real *src, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        dst[i] = (double)src[i];
}

/* h: [M][d] input rows (embeddings), overwritten with h^(L).  Row i sits at
   position P+i, sees cached positions 0..P-1 and rows 0..i. */
static void forward_rows(eo_session *s, real *h, int P, int M, const head_req *hr,
                         const eo_trace *tr)
{
    const eo_model *m = s->m;
    const int d = m->c.d_model, H = m->c.n_heads, hd = m->c.head_dim, F = m->c.d_ffn,
              V = m->c.vocab, L = m->c.n_layers;
    const real eps = (real)m->c.rms_eps;
    const real scale = (real)(1.0 / sqrt((double)hd));
    size_t Md = (size_t)M * d;
    real *x = (real *)malloc(Md * sizeof(real));
    real *q = (real *)malloc(Md * sizeof(real));
    real *k = (real *)malloc(Md * sizeof(real));
    real *v = (real *)malloc(Md * sizeof(real));
    real *att = (real *)malloc(Md * sizeof(real));
    real *o = (real *)malloc(Md * sizeof(real));
    real *gate = (real *)malloc((size_t)M * F * sizeof(real));
    real *up = (real *)malloc((size_t)M * F * sizeof(real));

    if (tr && tr->h) copy_trace(tr->h, h, Md);
    for (int l = 1; l <= L; ++l) {
        const layer_w *w = &m->layers[l - 1];
        real *kc = s->kc + (size_t)(l - 1) * s->max_ctx * d;
        real *vc = s->vc + (size_t)(l - 1) * s->max_ctx * d;

        /* attention block */
        rmsnorm(h, w->g_attn, M, d, eps, x);
        linear(w->wq, d, d, x, M, q);
        linear(w->wk, d, d, x, M, k);
        linear(w->wv, d, d, x, M, v);
#pragma omp parallel for schedule(static)
        for (int i = 0; i < M; ++i) {
            rope_row(q + (size_t)i * d, H, hd, P + i, (double)m->c.rope_base);
            rope_row(k + (size_t)i * d, H, hd, P + i, (double)m->c.rope_base);
            memcpy(kc + (size_t)(P + i) * d, k + (size_t)i * d, (size_t)d * sizeof(real));
            memcpy(vc + (size_t)(P + i) * d, v + (size_t)i * d, (size_t)d * sizeof(real));
        }
        if (tr && tr->q) copy_trace(tr->q + (size_t)(l - 1) * Md, q, Md);
        if (tr && tr->k) copy_trace(tr->k + (size_t)(l - 1) * Md, k, Md);
        if (tr && tr->v) copy_trace(tr->v + (size_t)(l - 1) * Md, v, Md);
#pragma omp parallel for collapse(2) schedule(static)
        for (int i = 0; i < M; ++i) {
            for (int hh = 0; hh < H; ++hh) {
                int n_pos = P + i + 1;
                real *sc = (real *)malloc((size_t)n_pos * sizeof(real));
                const real *qi = q + (size_t)i * d + (size_t)hh * hd;
                for (int t = 0; t < n_pos; ++t)
                    sc[t] = dot_rr(qi, kc + (size_t)t * d + (size_t)hh * hd, hd) * scale;
                softmax_inplace(sc, n_pos);
                real *out = att + (size_t)i * d + (size_t)hh * hd;
                for (int e = 0; e < hd; ++e)
                    out[e] = 0;
                for (int t = 0; t < n_pos; ++t) {
                    const real *vt = vc + (size_t)t * d + (size_t)hh * hd;
                    for (int e = 0; e < hd; ++e)
                        out[e] += sc[t] * vt[e];
                }
                free(sc);
            }
        }
        if (tr && tr->attn) copy_trace(tr->attn + (size_t)(l - 1) * Md, att, Md);
        linear(w->wo, d, d, att, M, o);
        for (size_t i = 0; i < Md; ++i)
            h[i] += o[i];

        /* SwiGLU block */
        rmsnorm(h, w->g_ffn, M, d, eps, x);
        linear(w->wg, F, d, x, M, gate);
        linear(w->wu, F, d, x, M, up);
        for (size_t i = 0; i < (size_t)M * F; ++i)
            gate[i] = silu(gate[i]) * up[i];
        linear(w->wd, d, F, gate, M, o);
        for (size_t i = 0; i < Md; ++i)
            h[i] += o[i];
        if (tr && tr->h) copy_trace(tr->h + (size_t)l * Md, h, Md);

        /* LM head on this layer's hidden state where requested */
        for (int e = 0; hr && e < hr->n_heads; ++e) {
            if (hr->layer[e] != l) continue;
            const int slot = l < L ? exit_slot(m, l) : -1;
            if (slot >= 0 && m->n_ad > 0) {
                adapter_rows(m, slot, h, M, o);
                rmsnorm(o, hr->gain[e], M, d, eps, x);
            } else {
                rmsnorm(h, hr->gain[e], M, d, eps, x);
            }
            linear(m->w_lm, V, d, x, M, hr->logits[e]);
        }
    }
    free(x); free(q); free(k); free(v); free(att); free(o); free(gate); free(up);
}

static void embed_tokens(const eo_model *m, const int32_t *tok, int n, real *h)
{
    int d = m->c.d_model;
    for (int i = 0; i < n; ++i)
        for (int kx = 0; kx < d; ++kx)
            h[(size_t)i * d + kx] = bf16_val(m->emb[(size_t)tok[i] * d + kx]);
}

static void embed_raw(const uint16_t *emb, int n, int d, real *h)
{
    for (size_t i = 0; i < (size_t)n * d; ++i)
        h[i] = bf16_val(emb[i]);
}

static int tokens_ok(const eo_model *m, const int32_t *t, int n)
{
    for (int i = 0; i < n; ++i)
        if (t[i] < 0 || t[i] >= m->c.vocab) return 0;
    return 1;
}

#define PREFILL_CHUNK 16

int eo_prefill_embeds(eo_session *s, const uint16_t *emb_bf16, int n_emb, const int32_t *tokens,
                      int n, unsigned flags, int32_t *first_token)
{
    if (!s || n_emb < 0 || n < 0 || (n_emb > 0 && !emb_bf16) || (n > 0 && !tokens))
        return EO_EINVAL;
    const eo_model *m = s->m;
    const int d = m->c.d_model, V = m->c.vocab;
    if (!tokens_ok(m, tokens, n)) return EO_EINVAL;
    int hold = (flags & EO_HOLD_LAST) != 0;
    if (hold && n < 1) return EO_EINVAL;
    int total = n_emb + n - (hold ? 1 : 0); /* rows whose KV gets cached */
    if (!hold && total < 1) return EO_EINVAL;
    if (total + 1 > s->max_ctx) return EO_ECAPACITY;

    s->kv_len = 0;
    s->last_M = 0;
    s->has_pending = 0;
    real *h = (real *)malloc((size_t)PREFILL_CHUNK * d * sizeof(real));
    real *logits = (real *)malloc((size_t)PREFILL_CHUNK * V * sizeof(real));
    for (int start = 0; start < total; start += PREFILL_CHUNK) {
        int M = total - start < PREFILL_CHUNK ? total - start : PREFILL_CHUNK;
        for (int i = 0; i < M; ++i) {
            int r = start + i;
            if (r < n_emb)
                embed_raw(emb_bf16 + (size_t)r * d, 1, d, h + (size_t)i * d);
            else
                embed_tokens(m, tokens + (r - n_emb), 1, h + (size_t)i * d);
        }
        int last = (start + M == total) && !hold;
        head_req hr;
        hr.n_heads = last ? 1 : 0;
        hr.layer[0] = m->c.n_layers;
        hr.gain[0] = m->g_final;
        hr.logits[0] = logits;
        forward_rows(s, h, start, M, &hr, NULL);
        if (last) {
            s->pending = argmax_lowest(logits + (size_t)(M - 1) * V, V);
            s->has_pending = 1;
            if (first_token) *first_token = s->pending;
        }
    }
    if (hold) {
        s->pending = tokens[n - 1];
        s->has_pending = 1;
    }
    s->kv_len = total;
    free(h);
    free(logits);
    return EO_OK;
}

int eo_prefill(eo_session *s, const int32_t *tokens, int n, unsigned flags, int32_t *first_token)
{
    return eo_prefill_embeds(s, NULL, 0, tokens, n, flags, first_token);
}

int eo_verify(eo_session *s, const int32_t *drafts, int gamma, const int32_t *exit_layers,
              int n_exits, int commit, eo_result *out, double *logits_out, const eo_trace *trace)
{
    if (!s || !out || !drafts) return EO_EINVAL;
    const eo_model *m = s->m;
    const int d = m->c.d_model, V = m->c.vocab, L = m->c.n_layers;
    if (gamma < 1 || gamma + 1 > EO_MAX_M) return EO_EINVAL;
    if (n_exits < 0 || n_exits > EO_MAX_EXITS || (n_exits > 0 && !exit_layers)) return EO_EINVAL;
    for (int e = 0; e < n_exits; ++e) {
        if (exit_layers[e] < 1 || exit_layers[e] > L - 1) return EO_EINVAL;
        if (e > 0 && exit_layers[e] <= exit_layers[e - 1]) return EO_EINVAL;
        if (!exit_gain(m, exit_layers[e])) return EO_EINVAL;
    }
    if (!tokens_ok(m, drafts, gamma)) return EO_EINVAL;
    if (!s->has_pending) return EO_ESTATE;
    const int M = gamma + 1, P = s->kv_len;
    if (P + M > s->max_ctx) return EO_ECAPACITY;

    int32_t rows[EO_MAX_M];
    rows[0] = s->pending;
    for (int j = 0; j < gamma; ++j)
        rows[j + 1] = drafts[j];

    real *h = (real *)malloc((size_t)M * d * sizeof(real));
    embed_tokens(m, rows, M, h);
    head_req hr;
    hr.n_heads = n_exits + 1;
    for (int e = 0; e < n_exits; ++e) {
        hr.layer[e] = exit_layers[e];
        hr.gain[e] = exit_gain(m, exit_layers[e]);
    }
    hr.layer[n_exits] = L;
    hr.gain[n_exits] = m->g_final;
    for (int e = 0; e <= n_exits; ++e)
        hr.logits[e] = (real *)malloc((size_t)M * V * sizeof(real));

    forward_rows(s, h, P, M, &hr, trace);

    memset(out, 0, sizeof *out);
    out->gamma = gamma;
    out->n_exits = n_exits;
    for (int e = 0; e <= n_exits; ++e) {
        int32_t *a = e < n_exits ? out->exit_tokens[e] : out->final_tokens;
        double *conf = e < n_exits ? out->exit_conf[e] : out->final_conf;
        for (int i = 0; i < M; ++i) {
            a[i] = argmax_lowest(hr.logits[e] + (size_t)i * V, V);
            conf[i] = max_softmax(hr.logits[e] + (size_t)i * V, V);
        }
        if (e < n_exits)
            accept_rule(drafts, gamma, a, &out->exit_accept_len[e], NULL);
        else
            accept_rule(drafts, gamma, a, &out->accept_len, &out->next_token);
        if (logits_out)
            copy_trace(logits_out + (size_t)e * M * V, hr.logits[e], (size_t)M * V);
    }
    s->last_P = P;
    s->last_M = M;
    if (commit) {
        s->kv_len = P + out->accept_len + 1;
        s->pending = out->next_token;
    }
    for (int e = 0; e <= n_exits; ++e)
        free(hr.logits[e]);
    free(h);
    return EO_OK;
}

/* ---------- brute force without a cache ---------- */

int eo_full_logits(const eo_model *m, const uint16_t *emb_bf16, int n_emb, const int32_t *tokens,
                   int n, int exit_layer, double *logits_out)
{
    if (!m || n_emb < 0 || n < 0 || n_emb + n < 1 || !logits_out) return EO_EINVAL;
    if (!tokens_ok(m, tokens, n)) return EO_EINVAL;
    const int d = m->c.d_model, H = m->c.n_heads, hd = m->c.head_dim, F = m->c.d_ffn,
              V = m->c.vocab;
    const int L_run = exit_layer == 0 ? m->c.n_layers : exit_layer;
    const uint16_t *gain = exit_layer == 0 ? m->g_final : exit_gain(m, exit_layer);
    if (!gain || L_run < 1 || L_run > m->c.n_layers) return EO_EINVAL;
    const int T = n_emb + n;
    const real eps = (real)m->c.rms_eps;
    const real scale = (real)(1.0 / sqrt((double)hd));
    size_t Td = (size_t)T * d;
    real *h = (real *)malloc(Td * sizeof(real));
    real *x = (real *)malloc(Td * sizeof(real));
    real *q = (real *)malloc(Td * sizeof(real));
    real *k = (real *)malloc(Td * sizeof(real));
    real *v = (real *)malloc(Td * sizeof(real));
    real *att = (real *)malloc(Td * sizeof(real));
    real *o = (real *)malloc(Td * sizeof(real));
    real *gate = (real *)malloc((size_t)T * F * sizeof(real));
    real *up = (real *)malloc((size_t)T * F * sizeof(real));
    real *sc = (real *)malloc((size_t)T * sizeof(real));
    if (n_emb) embed_raw(emb_bf16, n_emb, d, h);
    if (n) embed_tokens(m, tokens, n, h + (size_t)n_emb * d);

    for (int l = 1; l <= L_run; ++l) {
        const layer_w *w = &m->layers[l - 1];
        rmsnorm(h, w->g_attn, T, d, eps, x);
        linear(w->wq, d, d, x, T, q);
        linear(w->wk, d, d, x, T, k);
        linear(w->wv, d, d, x, T, v);
        for (int t = 0; t < T; ++t) {
            rope_row(q + (size_t)t * d, H, hd, t, (double)m->c.rope_base);
            rope_row(k + (size_t)t * d, H, hd, t, (double)m->c.rope_base);
        }
        /* causal attention over the whole sequence: row t sees rows 0..t */
        for (int t = 0; t < T; ++t) {
            for (int hh = 0; hh < H; ++hh) {
                const real *qt = q + (size_t)t * d + (size_t)hh * hd;
                for (int u = 0; u <= t; ++u)
                    sc[u] = dot_rr(qt, k + (size_t)u * d + (size_t)hh * hd, hd) * scale;
                softmax_inplace(sc, t + 1);
                real *out = att + (size_t)t * d + (size_t)hh * hd;
                for (int e = 0; e < hd; ++e) {
                    real acc = 0;
                    for (int u = 0; u <= t; ++u)
                        acc += sc[u] * v[(size_t)u * d + (size_t)hh * hd + e];
                    out[e] = acc;
                }
            }
        }
        linear(w->wo, d, d, att, T, o);
        for (size_t i = 0; i < Td; ++i)
            h[i] += o[i];
        rmsnorm(h, w->g_ffn, T, d, eps, x);
        linear(w->wg, F, d, x, T, gate);
        linear(w->wu, F, d, x, T, up);
        for (size_t i = 0; i < (size_t)T * F; ++i)
            gate[i] = silu(gate[i]) * up[i];
        linear(w->wd, d, F, gate, T, o);
        for (size_t i = 0; i < Td; ++i)
            h[i] += o[i];
    }
    if (exit_layer != 0 && m->n_ad > 0) {
        adapter_rows(m, exit_slot(m, exit_layer), h, T, o);
        rmsnorm(o, gain, T, d, eps, x);
    } else {
        rmsnorm(h, gain, T, d, eps, x);
    }
    real *z = (real *)malloc((size_t)T * V * sizeof(real));
    linear(m->w_lm, V, d, x, T, z);
    copy_trace(logits_out, z, (size_t)T * V);
    free(z); free(h); free(x); free(q); free(k); free(v); free(att); free(o);
    free(gate); free(up); free(sc);
    return EO_OK;
}

int eo_ar_decode(const eo_model *m, const uint16_t *emb_bf16, int n_emb, const int32_t *tokens,
                 int n, int exit_layer, int n_new, int32_t *out_tokens)
{
    if (!m || n_new < 0 || !out_tokens) return EO_EINVAL;
    const int V = m->c.vocab;
    int32_t *seq = (int32_t *)malloc((size_t)(n + n_new) * sizeof(int32_t));
    memcpy(seq, tokens, (size_t)n * sizeof(int32_t));
    double *z = (double *)malloc((size_t)(n_emb + n + n_new) * V * sizeof(double));
    int rc = EO_OK;
    for (int j = 0; j < n_new; ++j) {
        int T = n_emb + n + j;
        rc = eo_full_logits(m, emb_bf16, n_emb, seq, n + j, exit_layer, z);
        if (rc != EO_OK) break;
        /* argmax in the oracle's own precision: the values were widened exactly */
        const double *zl = z + (size_t)(T - 1) * V;
        int best = 0;
        for (int i = 1; i < V; ++i)
            if (zl[i] > zl[best]) best = i;
        seq[n + j] = best;
        out_tokens[j] = best;
    }
    free(z);
    free(seq);
    return rc;
}
