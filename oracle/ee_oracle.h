/*
 * CPU oracle for the server-side verification pass of speculative edge-cloud
 * decoding with early exits.  TEST INFRASTRUCTURE ONLY: nothing in the product
 * path may include, link or call this.  It shares no code with the GPU library;
 * it has its own model-file reader and its own arithmetic.
 *
 * What it computes (paper: Background, Eq. 2 "Verify"; Eq. 3 layer recurrence
 * and the per-layer LM head; Methodology Step 2, Eq. 5 multi-exit Verify;
 * Appendix "System Design", server LISTENER's VERIFY call):
 *   one forward pass of a Llama-style decoder over the rows
 *   [pending, draft_1 .. draft_gamma]; at every requested exit layer and at the
 *   last layer, the LM head's argmax token per row, the number of accepted
 *   drafts (longest prefix with draft_{j} == argmax at row j-1) and the token
 *   generated after the accepted prefix.
 * Verification is greedy exact-match (temperature-0 case of the paper's
 * criterion); ties in the argmax go to the lowest token id.
 *
 * Arithmetic type: EO_REAL (float unless the library is built with
 * -DEO_REAL=double).  Weights are the bf16 values of the model file, widened
 * exactly.  The KV cache holds EO_REAL values (no rounding).
 *
 * Pins (tests/test_oracle_*.py): brute-force token-by-token decoding without a
 * cache, closed-form special cases, library routines of PyTorch-CPU in float64,
 * invariants of RoPE and of the accept rule.  No values printed by the paper
 * exist for this path.
 */
#ifndef EE_ORACLE_H
#define EE_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EO_MAX_EXITS 40
#define EO_MAX_M 64

#define EO_OK 0
#define EO_EINVAL (-1)
#define EO_ESTATE (-2)
#define EO_ECAPACITY (-3)
#define EO_EIO (-4)
#define EO_EFORMAT (-5)

#define EO_HOLD_LAST 1u

typedef struct eo_model eo_model;
typedef struct eo_session eo_session;

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab, n_exits;
    float rope_base, rms_eps;
    int32_t exit_layers[EO_MAX_EXITS];
} eo_config;

typedef struct {
    int32_t gamma, n_exits;
    int32_t accept_len;                              /* delta in [0, gamma]              */
    int32_t next_token;                              /* final_tokens[accept_len]         */
    int32_t final_tokens[EO_MAX_M];                  /* final-head argmax at rows 0..gamma */
    int32_t exit_accept_len[EO_MAX_EXITS];           /* delta^(e)                         */
    int32_t exit_tokens[EO_MAX_EXITS][EO_MAX_M];     /* exit-head argmax at rows 0..gamma */
    /* confidence score of every row (paper Eq. 4): max over the vocabulary of softmax(z) */
    double final_conf[EO_MAX_M];
    double exit_conf[EO_MAX_EXITS][EO_MAX_M];
} eo_result;

/* Optional per-stage capture for kernel-level comparisons; any pointer may be
   NULL.  Shapes use M = number of rows of the pass, d = d_model, L = n_layers.
   All buffers are double regardless of EO_REAL. */
typedef struct {
    double *h;      /* [(L+1)][M][d]  residual stream: h^(0) .. h^(L)             */
    double *q;      /* [L][M][d]      queries after RoPE                           */
    double *k;      /* [L][M][d]      keys after RoPE (as cached)                  */
    double *v;      /* [L][M][d]      values (as cached)                           */
    double *attn;   /* [L][M][d]      attention output before the output projection */
} eo_trace;

int eo_sizeof_real(void);

int eo_model_open(const char *path, eo_model **out);
void eo_model_close(eo_model *m);
int eo_model_config(const eo_model *m, eo_config *out);

int eo_session_new(const eo_model *m, int max_ctx, eo_session **out);
void eo_session_free(eo_session *s);

/* Caches KV for n prompt tokens and sets pending = argmax of the final head at
   the last prompt row (returned in *first_token).  With EO_HOLD_LAST: caches
   n-1 tokens, pending = tokens[n-1], *first_token untouched. */
int eo_prefill(eo_session *s, const int32_t *tokens, int n, unsigned flags, int32_t *first_token);
/* Same with n_emb rows of bf16[d] (raw uint16) placed before the n tokens. */
int eo_prefill_embeds(eo_session *s, const uint16_t *emb_bf16, int n_emb, const int32_t *tokens,
                      int n, unsigned flags, int32_t *first_token);

/* One verification pass over [pending, drafts[0..gamma-1]].
   exit_layers: n_exits strictly increasing values in [1, L-1], each with a stored gain.
   logits_out: NULL, or double[(n_exits+1)][gamma+1][V] (exit heads in order, final last).
   commit != 0: kv_len += accept_len+1, pending = next_token. */
int eo_verify(eo_session *s, const int32_t *drafts, int gamma, const int32_t *exit_layers,
              int n_exits, int commit, eo_result *out, double *logits_out, const eo_trace *trace);

int eo_kv_truncate(eo_session *s, int new_len);
/* after eo_verify(commit = 0): kv_len = (position of that pass) + delta + 1, pending = token */
int eo_commit_rows(eo_session *s, int delta, int32_t token);
int eo_set_pending(eo_session *s, int32_t token);
int eo_kv_len(const eo_session *s);
int eo_pending(const eo_session *s, int32_t *token);

/* Brute force, no cache object: logits of head `exit_layer` (0 = final head after
   layer L, e>0 = exit head after layer e) for every row of a sequence made of
   n_emb embedding rows followed by n tokens, recomputed from scratch.
   logits_out: double[n_emb+n][V]. */
int eo_full_logits(const eo_model *m, const uint16_t *emb_bf16, int n_emb, const int32_t *tokens,
                   int n, int exit_layer, double *logits_out);

/* Brute-force greedy autoregressive decoding: n_new tokens, each from a
   from-scratch forward over the whole sequence so far (eo_full_logits). */
int eo_ar_decode(const eo_model *m, const uint16_t *emb_bf16, int n_emb, const int32_t *tokens,
                 int n, int exit_layer, int n_new, int32_t *out_tokens);

#ifdef __cplusplus
}
#endif
#endif
