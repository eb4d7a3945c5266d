/*
 * libeeverify -- server-side target-model verification pass with early exits
 * for speculative edge-cloud decoding, for AMD MI355X (gfx950).
 *
 * One call of ee_verify runs ONE forward pass of a Llama-style decoder over the
 * rows [pending, draft_1 .. draft_gamma] (the gamma drafted tokens plus one).
 * After each requested intermediate layer an exit head (RMSNorm with that
 * exit's gain, then the shared LM head) yields the argmax token of every row
 * and that exit's accept length; these are written to pinned host memory and a
 * hipEvent is recorded, so the caller can read them while the pass is still
 * running.  After the last layer the final head gives the accept length, the
 * correction/bonus token and the KV-cache rollback.
 *
 * Paper passages the operations follow:
 *   - Verify: Background, Eq. 2 (target accepts delta <= gamma drafts and
 *     produces one more token; the prefix then grows by delta+1).
 *   - Layer recurrence h^(l) = f^(l)(h^(l-1)) and per-layer LM head
 *     z^(l) = LMHead(h^(l)): Background "Early Exit in LLMs", Eq. 3.
 *   - Every exit verifies the drafts on its own logits: Methodology Step 2, Eq. 5.
 *   - Exit results leave the server as soon as they exist: Methodology Step 3;
 *     Appendix "System Design", server LISTENER/SENDER (Algorithm 2).
 * Exit heads: RMSNorm with the exit's gain, then the shared LM head; when the model file carries
 * adapters (the paper's "adapter layers after each layer" that connect a layer to the LM head;
 * Methodology, early-exit fine-tuning), the layer's output first goes through them:
 *   a = h + sum_j (W_up,j silu(W_down,j h + b_down,j) + b_up,j)   (bottlenecks in parallel),
 * and the head is evaluated on a.  The final head has no adapter.
 * Verification is greedy exact-match (the temperature-0 case of the paper's
 * criterion): draft j is accepted iff it equals the argmax at row j-1 and all
 * earlier drafts were accepted.  Argmax ties go to the lowest token id.
 * The KV cache and its rollback are this library's (the paper's server is
 * handed the whole prefix every round).
 *
 * Conventions
 *   - All pointers in the signatures are HOST pointers.  Device memory is owned
 *     by the library.  Input arrays belong to the caller and are copied before
 *     the call returns.
 *   - Every function returns an int status: EE_OK (0) or a negative EE_E* code;
 *     ee_last_error() gives a thread-local message for the last failure.
 *     Nothing throws, nothing aborts.
 *   - A session is not thread-safe.  A model may be shared by sessions used
 *     from different threads, but passes of sessions of one model must not
 *     overlap in time on the GPU unless they run in one ee_verify_batch call.
 *   - Arithmetic: bf16 weights and KV cache, bf16 MFMA operands with fp32
 *     accumulation, fp32 residual stream / norms / softmax.
 */
#ifndef EE_H
#define EE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EE_MAX_M 16      /* rows per session and pass: gamma + 1 <= EE_MAX_M          */
#define EE_MAX_EXITS 40  /* exit heads per pass (the paper runs 31 / 39: one after every layer but the last) */
#define EE_MAX_BATCH 16  /* sessions per ee_verify_batch                              */
#define EE_MAX_ROWS 48   /* rows per pass over all sessions of a batch                */

#define EE_OK 0
#define EE_NOT_READY 1        /* ee_query_*, ee_exit_pop: the result is not there yet  */
#define EE_DONE 2             /* ee_exit_pop: nothing left to send for this pass       */
#define EE_EINVAL (-1)        /* bad argument                                          */
#define EE_ESTATE (-2)        /* call not allowed in this state                        */
#define EE_ECAPACITY (-3)     /* kv_len + gamma + 1 would exceed max_ctx               */
#define EE_EIO (-4)           /* model file cannot be read                             */
#define EE_EFORMAT (-5)       /* model file is not in the expected format              */
#define EE_EDEVICE (-6)       /* HIP error or device-side failure (see ee_last_error)  */

/* ee_prefill flags */
#define EE_HOLD_LAST 1u       /* cache n-1 tokens, pending = tokens[n-1], no logits     */
/* ee_session_create flags */
#define EE_KEEP_LOGITS 1u     /* keep every head's logits of the last pass (debug)      */
#define EE_NO_AUTOCOMMIT 2u   /* final accept does not move kv_len / pending            */
#define EE_SAMPLING 4u        /* the session can run ee_verify_sampled: it holds device room for
                                 max_gamma draft distributions and for the heads' logits      */
#define EE_TIME_LAUNCHES 16u  /* measurement: an event pair around every launch of a verify
                                 pass (see ee_launch_times); perturbs the pass slightly    */

typedef struct ee_model ee_model;     /* opaque; immutable after load                   */
typedef struct ee_session ee_session; /* opaque; one KV cache, one stream               */

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int32_t n_exits;                       /* exit gains stored in the model            */
    int32_t exit_layers[EE_MAX_EXITS];     /* 1-based: exit e sits after layer e        */
    float rope_base, rms_eps;
    int32_t n_adapters, adapter_width;     /* bottleneck adapters per exit head and their width
                                              (0: exit heads are RMSNorm + LM head only)  */
    int32_t max_rows;                      /* rows per pass this instance was laid out for */
    int32_t n_workgroups;                  /* persistent grid size (= compute units)    */
} ee_model_config;

/* Result block of one pass; lives in pinned host memory owned by the session and
   stays valid until the next ee_verify / ee_verify_batch / ee_prefill on it.
   exit_tokens[e], exit_accept_len[e]: readable after ee_wait_exit(e) or
   ee_query_exit(e) == EE_OK.  The other fields: after ee_wait_final.
   The paper's exit message x^(e)_{t:t+delta^(e)+1} is
   draft[0 .. delta^(e)-1] followed by exit_tokens[e][delta^(e)]. */
typedef struct {
    int32_t gamma, n_exits;
    int32_t accept_len;                             /* delta in [0, gamma]              */
    int32_t next_token;                             /* final_tokens[accept_len]         */
    int32_t final_tokens[EE_MAX_M];                 /* final-head argmax, rows 0..gamma */
    int32_t exit_accept_len[EE_MAX_EXITS];          /* delta^(e)                        */
    int32_t exit_tokens[EE_MAX_EXITS][EE_MAX_M];    /* exit-head argmax, rows 0..gamma  */
    int32_t device_status;                          /* 0, or != 0 if a device-side wait
                                                       gave up (pass result invalid)    */
    int32_t reserved[15];
    /* Confidence score of every row (paper Eq. 4): the largest entry of softmax(z) of the head's
       logits, the value the paper's sender and client queues order exit results by.  Readable
       together with the tokens of the same head. */
    float final_conf[EE_MAX_M];
    float exit_conf[EE_MAX_EXITS][EE_MAX_M];
} ee_verify_result;

const char *ee_last_error(void);

/* Reads a model file (header + row-major bf16 tensors, see the generator's
   format description), uploads it to GPU `device` and re-lays the weight
   matrices out in the tile order the kernels stream.  max_rows (1..EE_MAX_ROWS)
   is the largest number of rows a pass (or a prefill chunk) will carry; ee_model_load
   uses 16.  With max_rows > 16 the output and down projections are kept in a second
   tile order as well, in which groups of four workgroups share their output columns and
   split K; launches of more than 16 rows use it (about a quarter more device memory for
   the weights).
   Cold path; synchronous. */
int ee_model_load(const char *path, int device, ee_model **out);
int ee_model_load_ex(const char *path, int device, int max_rows, ee_model **out);

/* Tuning and test knob, process-wide, for models loaded after the call with max_rows > 16:
   which GEMM kinds get the K-split tile order (kind_mask: bit 0 QKV, 1 output projection,
   2 gate/up, 3 down projection, 4 LM head, 5 and 6 the adapters; default output and down)
   and into how many workgroups K is split (2^log2_splits, 1 <= log2_splits <= 3; default 2).
   A kind whose K is not a multiple of 32 * 2^log2_splits stays unsplit.  Results are the
   same up to the order of the fp32 sums.  Not synchronised with concurrent loads.
   EE_EINVAL for values outside these ranges. */
int ee_tune_k_split(unsigned kind_mask, int log2_splits);
int ee_model_free(ee_model *m);
int ee_model_info(const ee_model *m, ee_model_config *out);

/* A session owns a paged bf16 KV cache for up to max_ctx positions, scratch
   for one pass, a stream, events and a pinned result block.
   max_gamma in [1, EE_MAX_M-1]. */
int ee_session_create(const ee_model *m, int max_ctx, int max_gamma, unsigned flags,
                      ee_session **out);
int ee_session_free(ee_session *s);

/* Prefill (synchronous): caches KV for all n prompt tokens, sets
   pending = *first_token = argmax of the final head at the last prompt row,
   kv_len = n.  With EE_HOLD_LAST (the paper's first round, where the drafts
   follow the prompt directly): kv_len = n-1, pending = tokens[n-1], no head is
   evaluated and *first_token is left alone.  Resets the session first.
   tokens: n ids in [0, vocab). */
int ee_prefill(ee_session *s, const int32_t *tokens, int n, unsigned flags, int32_t *first_token);
/* Same, with n_emb rows of bf16[d_model] (raw uint16, row-major) placed before
   the n tokens: the image-patch-prefix-then-text structure of the paper's
   vision-language experiment. */
int ee_prefill_embeds(ee_session *s, const uint16_t *emb_bf16, int n_emb, const int32_t *tokens,
                      int n, unsigned flags, int32_t *first_token);

/* Asynchronous: enqueues one pass over [pending, draft_tokens[0..gamma-1]] and
   returns.  exit_layers: n_exits strictly increasing values in [1, L-1], each
   with a stored exit gain.  *out (may be NULL) receives the session's result
   block.  A pass still in flight on this session is waited for first. */
int ee_verify(ee_session *s, const int32_t *draft_tokens, int gamma, const int32_t *exit_layers,
              int n_exits, const ee_verify_result **out);
/* One pass for several sessions of one model (multi-client serving, the paper's
   batch-processing appendix): every weight byte is streamed once for all rows of all
   sessions; attention, accept and rollback are per session.  The first session leads
   the pass: its stream, events and scratch carry it (list the session with the largest
   max_ctx first); every session's own result block is filled and every session can be
   waited on.  drafts[i] has gamma ids; n_sessions * (gamma+1) must not exceed the
   model's max_rows (at most EE_MAX_ROWS).  outs may be NULL. */
int ee_verify_batch(ee_session *const *sessions, int n_sessions, const int32_t *const *drafts,
                    int gamma, const int32_t *exit_layers, int n_exits,
                    const ee_verify_result **outs);

/* ee_verify for callers that cannot allocate GPU memory: code under HIP graph capture, tight
   serving loops, harnesses that forbid hipMalloc.  Same pass, same results; the pass's scratch
   (residual stream, GEMM inputs, norm partials, attention partials, argmax candidates, counters)
   lives in a static device array of EE_STATIC_SCRATCH_BYTES that every GPU the library runs on
   holds until the process ends, instead of in the session's own buffers.  Neither this call nor
   anything it runs calls hipMalloc / hipFree or an allocating library routine.  One session per
   call; EE_ECAPACITY if gamma + 1 rows of this model (or the context's attention partials) do not
   fit the array; not for EE_TIME_LAUNCHES sessions.  Calls on one GPU share that GPU's array: two
   ee_verify_static passes must not overlap in time on a GPU (wait for one before the next, also
   across sessions); passes enqueued with ee_verify / ee_verify_batch are not affected.  Inputs,
   the KV cache and the pinned result block are the session's as usual. */
#define EE_STATIC_SCRATCH_BYTES (8 << 20)
int ee_verify_static(ee_session *s, const int32_t *draft_tokens, int gamma, const int32_t *exit_layers,
                     int n_exits, const ee_verify_result **out);

/* Probabilistic verification: VERIFY with the draft model's probability distributions
   (paper: Background Eq. 2, Methodology Step 2 Eq. 5, Appendix "System Design" Alg. 2
   LISTENER, which all pass p to VERIFY; the criterion is that of the speculative sampling
   scheme the paper builds on).  Same pass as ee_verify; every head (exits and final) decides
   with its own logits z:  q_i = softmax(z_i / temperature) at row i;  draft i+1 (token x) is
   kept iff u[i] * p_i(x) < q_i(x);  if the round ends at row i < gamma, the row emits the first
   token k (in id order) with  sum_{j<=k} w_j > v[i] * sum_j w_j,  w = max(q_i - p_i, 0)  (w = q_i
   if that is zero everywhere);  row gamma emits the same with w = q_gamma.  accept_len /
   exit_accept_len = the drafts kept before the first one that is not; final_tokens[i] /
   exit_tokens[e][i] = the token row i emits if the round ends there; next_token =
   final_tokens[accept_len]; the confidences are those of ee_verify (Eq. 4 on the logits as
   they are).  Emitted tokens are then distributed as if the target model had sampled them at
   that temperature.  The random numbers are the caller's: every head uses the same u and v.
   All pointers are host memory, read before the call returns:
     draft_probs  [gamma][vocab] fp32, row i = the distribution draft i+1 was drawn from;
     u            [gamma] in [0,1);   v  [gamma+1] in [0,1);   temperature > 0.
   The cumulative sums are taken in 40-bit fixed point (exact, order-free), the probabilities
   in fp32.  Sessions created with EE_SAMPLING; gamma <= their max_gamma.
   ee_verify_sampled_batch is ee_verify_batch with samplings[i] for sessions[i] (each session
   its own distributions, numbers and temperature; every head of every session decides by the
   same rule).  The draft distributions travel to the device with the call: gamma * vocab
   floats per session. */
typedef struct ee_sampling {
    const float *draft_probs;
    const float *u;
    const float *v;
    float temperature;
} ee_sampling;
int ee_verify_sampled(ee_session *s, const int32_t *draft_tokens, int gamma, const int32_t *exit_layers,
                      int n_exits, const ee_sampling *sampling, const ee_verify_result **out);
int ee_verify_sampled_batch(ee_session *const *sessions, int n_sessions, const int32_t *const *drafts,
                            int gamma, const int32_t *exit_layers, int n_exits,
                            const ee_sampling *samplings, const ee_verify_result **outs);

int ee_wait_exit(ee_session *s, int exit_idx);   /* blocks until exit exit_idx is published */
int ee_query_exit(ee_session *s, int exit_idx);  /* EE_OK or EE_NOT_READY                   */
int ee_wait_final(ee_session *s);                /* blocks until the pass has finished      */
int ee_query_final(ee_session *s);

/* The server's SENDER side of the paper (Appendix "System Design", Algorithm 2): exit results
   wait in a queue Q_e and leave it in the order of their confidence score, because the
   network is slower than the exits are produced.  The score of exit e is
   s^(e) = max over rows 0..delta^(e) of the row's largest softmax probability (Alg. 2's
   max(q^(e)_{1:delta+1}) with Eq. 4's confidence), i.e. of exit_conf[e][0..exit_accept_len[e]].
   ee_exit_pop: among the exits of the pass in flight that are published and not popped yet,
   returns the one with the highest score (ties: the earlier exit) in *exit_idx / *score
   (EE_OK).  Nothing published: waits for the next exit if `wait`, else EE_NOT_READY.  EE_DONE
   when every exit has been popped or the final result is there (Alg. 2 resets the queue when
   the final result is sent).  Host-side only: polls the exit events.
   ee_exit_order: after the pass has finished, all its exits in the order the queue would
   release them if all were waiting (score descending); order / scores have n_exits entries. */
int ee_exit_pop(ee_session *s, int wait, int *exit_idx, float *score);
int ee_exit_order(ee_session *s, int *order, float *scores);

/* The paper's latency model (Experiments, table "Latency calculation"; notation table) and
   its speed-up projection (Appendix "Speedup Projection Analysis", Eq. 9), fed with measured
   times.  All times in milliseconds.
     cloud autoregressive (AR):      2 T_c + n T_q
     edge-cloud speculative (SD):    (n / tau) (2 T_c + gamma T_p + T_q)
     with early exits (FSD):         (n / tau) (2 T_c + r gamma T_p + (1 - r) T_r + T_q)
     c = T_p / T_q;  projected SD -> FSD speed-up (T_c = T_r = 0):  (gamma c + 1) / (r gamma c + 1)
   EE_EINVAL for non-positive tau, T_q or n, gamma < 1, r outside [0, 1] or negative times.
   Pure host arithmetic (double); needs no GPU. */
typedef struct {
    double T_p;   /* one forward pass of the draft model                          */
    double T_q;   /* one forward pass (verify pass) of the target model           */
    double T_c;   /* client <-> server communication latency, one way             */
    double T_r;   /* thread synchronisation latency on a pre-draft cache hit      */
    double tau;   /* tokens per draft-verify round: accepted + 1                  */
    double r;     /* pre-draft cache miss rate                                    */
    int32_t gamma, n;
} ee_latency_params;
typedef struct {
    double ar_ms, sd_ms, fsd_ms;                       /* n tokens                  */
    double ar_ms_per_token, sd_ms_per_token, fsd_ms_per_token;
    double speedup_ar_to_sd, speedup_sd_to_fsd;
    double c;                                          /* latency ratio T_p / T_q   */
    double projected_sd_to_fsd;                        /* Eq. 9                     */
} ee_latency;
int ee_latency_model(const ee_latency_params *p, ee_latency *out);

/* Milliseconds of GPU time from the start of the last pass to exit exit_idx's
   event (exit_idx in [0, n_exits)) or to the final event (exit_idx == n_exits).
   The pass must have finished. */
int ee_pass_time_ms(ee_session *s, int exit_idx, float *ms);

/* KV rollback / external commit: new_len <= kv_len; pages wholly beyond
   new_len return to the session's free list. */
int ee_kv_truncate(ee_session *s, int new_len);
int ee_set_pending(ee_session *s, int32_t token);
int ee_kv_len(ee_session *s, int *out);
int ee_pending(ee_session *s, int32_t *out);

/* Debug: logits of head head_idx of the last verify pass (0..n_exits-1 = exit heads in
   order, n_exits = final head) for this session's rows as float[gamma+1][vocab].  The
   session that led the pass (the session itself for ee_verify, the first one of an
   ee_verify_batch call) must have been created with EE_KEEP_LOGITS. */
int ee_debug_logits(ee_session *s, int head_idx, float *out);

/* Measurement aid: `reps` launches of a plain copy kernel (ee_copy_kernel) that moves `bytes`
   bytes each between two device buffers it allocates and frees: under the profiler's HBM
   traffic counters this is the reading of a known number of bytes read and written. */
int ee_debug_copy(int device, size_t bytes, int reps);

/* hipDeviceSynchronize on `device`: every pass enqueued so far has finished. */
int ee_device_synchronize(int device);

/* Per-session options; the session must have no pass in flight.
   EE_OPT_ATT_SPLITS: parts the cached positions of a head are split into for attention
     (1..16), 0 = chosen per pass from the context length and the number of compute units
     (the default).  A value the context or the scratch cannot take is raised / lowered to
     the nearest that works.
   EE_OPT_SCATTER_PAGES: 1 = hand KV pages out in descending order from the next ee_prefill
     on, so that the pages of a session are not consecutive and every lookup goes through the page
     table (the pages of a fresh session are consecutive and the kernels then skip the lookup).
   EE_OPT_HEAD_BATCH: exit heads evaluated by one launch of the LM head (default 1).  With k > 1
     every exit still deposits its head input when its layer is done, but the LM head matrix is
     streamed once for k consecutive exits (as many as the max_rows of the model allow) and their
     results are published together after the last of them: less traffic when many exits are
     active (the paper runs one after every layer), later results for the earlier exits of a
     group. */
#define EE_OPT_ATT_SPLITS 1
#define EE_OPT_SCATTER_PAGES 2
#define EE_OPT_HEAD_BATCH 3
int ee_session_option(ee_session *s, int option, int value);

/* Measurement (EE_TIME_LAUNCHES sessions, pass led by `s`): for every kernel launch of the
   last verify pass, in launch order, what it ran (EE_LAUNCH_* code) and the milliseconds
   between the HIP events recorded on the session's stream right before and right after
   it.  Waits for the pass.  Writes min(n, max_launches) entries to the host arrays. */
#define EE_LAUNCH_QKV 0     /* attention-norm + Q/K/V projection + RoPE + KV write       */
#define EE_LAUNCH_O 1       /* attention output projection + residual + FFN norm input   */
#define EE_LAUNCH_GU 2      /* gate/up projections + SiLU * up                           */
#define EE_LAUNCH_DN 3      /* down projection + residual + next norm inputs             */
#define EE_LAUNCH_HEAD 4    /* exit or final head: norm + LM head + argmax, accept rule,
                               publication, KV commit                                    */
#define EE_LAUNCH_ADAPTER_DOWN 5 /* exit-head adapters: hidden units                     */
#define EE_LAUNCH_ADAPTER_UP 6   /* exit-head adapters: output + residual + head norm input */
#define EE_LAUNCH_ATT 8     /* attention over the paged KV cache                         */
#define EE_LAUNCH_EMBED 7   /* embedding gather                                          */
#define EE_LAUNCH_SAMPLE 9  /* ee_verify_sampled: keep tests and draws of a head's rows, accept
                               rule, publication, KV commit                              */
int ee_launch_times(ee_session *s, int32_t *codes, float *ms, int max_launches, int *n_launches);

/* Debug: runs one v_mfma_f32_16x16x32_bf16 through the operand lane layout the
   kernels assume and compares with the plain 16x32 . 32x16 product. */
int ee_debug_mfma_layout(int device);

/* Debug: the kernels divide small integers by run-time values (rows, workgroups, head size)
   with one reciprocal and one multiply.  Counts, on the device, the x in [0, 2 500 000]
   (the range the model loader admits) for which that differs from x / d, for each of the n
   divisors (host array, each >= 1, n <= 65536); *mismatches must come back 0. */
int ee_debug_div_small(int device, const int32_t *divisors, int n, long long *mismatches);

#ifdef __cplusplus
}
#endif
#endif
