/*
 * sd.h - C ABI of the draft-then-verify hot path of speculative decoding on one
 * AMD MI355X (gfx950).  Every step of the path runs in HIP kernels of this
 * library; there is no CPU fallback.
 *
 * Paper: arXiv 2505.08600.  Section 1 / Figure 1 define the two phases (a draft
 * model decodes gamma candidates autoregressively; the target model scores them in
 * one parallel pass), Section 2.1 / 2.4 the routing of a prompt to one of several
 * heterogeneous drafts, Section 3.1 the verification rule (speculative sampling;
 * greedy decoding as its argmax limit) and the LLaMA model family.
 *
 * State convention.  A context (sd_ctx) holds B sequences.  Sequence b has tokens
 * x_0..x_{n-1} in a device buffer of fixed capacity.  For every model attached to
 * the context there is a KV cache; the target's covers positions [0, n-1) between
 * calls (the last token is "pending": it is fed by the next verify), a draft's
 * covers [0, m) with m <= n-1.  All per-sequence lengths live in device memory, so
 * the draft -> verify -> draft loop needs no host synchronisation.
 *
 * Conventions for every call:
 *   - returns SD_OK (0) or a negative sd_status; sd_last_error() gives the text of
 *     the calling thread's last failure.  Nothing throws or aborts.
 *   - "dev" pointers are device memory owned by the caller and must stay valid
 *     until the work queued on `stream` has finished; "host" pointers are read
 *     before the call returns.
 *   - `stream` is a hipStream_t (NULL = the default stream).  sd_draft, sd_verify,
 *     sd_commit and sd_route only enqueue work; they never synchronise.
 *   - a model owns one activation workspace: at most one forward of a given model
 *     may be in flight at a time (calls on one stream are naturally ordered).
 *   - seq_ids (dev, int32[n_seq], or NULL for 0..n_seq-1) selects the sequences of
 *     the context a call works on; ids must be distinct.  1 <= n_seq <= the context's
 *     sequence count: an empty batch is SD_EINVAL, not a no-op.
 */
#ifndef SD_H
#define SD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sd_model sd_model; /* opaque: one target or draft model */
typedef struct sd_ctx sd_ctx;     /* opaque: B sequences, their tokens and KV caches */

typedef enum {
    SD_OK = 0,
    SD_EINVAL = -1, /* null pointer, bad shape, unsupported configuration */
    SD_ECAP = -2,   /* rows, gamma, batch or sequence capacity exceeded */
    SD_EHIP = -3,   /* HIP runtime failure; text in sd_last_error() */
    SD_ESTATE = -4  /* device-side consistency flag raised (see sd_ctx_sync) */
} sd_status;

enum { SD_FP32 = 0, SD_BF16 = 1 };

/* LLaMA-style decoder shape (Section 3.1 "Models"): pre-norm blocks with RMSNorm,
 * rotary embedding (rotate-half pairing, angle pos * rope_base^(-2i/head_dim)),
 * multi-head causal attention (n_kv_heads == n_heads), SwiGLU FFN, untied LM head,
 * no biases.  n_heads * head_dim must equal d_model; head_dim is 16, 32, 64 or 128 (the
 * matrix-core attention kernels take 64 and 128, the others run on the plain kernels);
 * vocab is a multiple of 4, at most 262144.
 * dtype SD_BF16: weights, the embedding table and the KV cache are bf16.  Every activation
 * that enters a contraction (normed hidden state, rotated query, attention output and
 * probabilities, SwiGLU product) is fed to the matrix cores as TWO bf16 terms, hi = bf16(x)
 * and lo = bf16(x - hi), i.e. about 16 mantissa bits: with single-bf16 activations two
 * correct implementations that add in different orders drift apart by more than the logit
 * tolerance over 32 layers.  Accumulation, the residual stream, softmax and logits are fp32.
 * (The normed hidden state is split into its two terms either after the division by rms or,
 * where option "norm_fold" applies, before it - the division then scales the fp32 sums.)
 * dtype SD_FP32: everything fp32.
 * max_rows: largest number of token rows one forward may carry
 *           (verify: n_seq * (gamma + 1); draft: 2 * n_seq; prefill chunks adapt).
 * max_pos : largest position + 1 (size of the rotary table). */
typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int32_t dtype;
    float rope_base, rms_eps;
    int32_t max_rows, max_pos;
} sd_model_config;

/* Device pointers to the weights, each matrix row-major [out][in] in the model's
 * dtype; RMSNorm gains are fp32 in both dtypes.  The per-layer members are HOST
 * arrays of n_layers DEVICE pointers.  sd_load_model copies every array into
 * memory the model owns (bf16 matrices are re-ordered into the tile order its
 * GEMM kernels stream), so the caller may release its buffers as soon as
 * sd_load_model has returned.  Matrices must be 16-byte aligned. */
typedef struct {
    const void *embed;         /* [vocab][d_model] */
    const void *lm_head;       /* [vocab][d_model] */
    const float *final_norm;   /* [d_model] */
    const void *const *wq;     /* [d_model][d_model] per layer */
    const void *const *wk;
    const void *const *wv;
    const void *const *wo;     /* [d_model][d_model] */
    const void *const *wgate;  /* [d_ffn][d_model] */
    const void *const *wup;    /* [d_ffn][d_model] */
    const void *const *wdown;  /* [d_model][d_ffn] */
    const float *const *norm_attn; /* [d_model] */
    const float *const *norm_ffn;  /* [d_model] */
} sd_weights;

/* Validate the configuration, copy the weights into the model's own device
 * memory (one allocation of about the size of the weights), build the rotary
 * table and allocate the activation workspace on the current device.
 * Synchronises.  SD_EINVAL on unsupported shapes, SD_EHIP if an allocation or
 * copy fails (nothing is leaked). */
int sd_load_model(const sd_model_config *cfg, const sd_weights *w, sd_model **out);
int sd_free_model(sd_model *m);

/* Low-rank adapters (Section 2.3: the heterogeneous drafts are LoRA fine-tunes of one base
 * model).  For the attention projections P in {q, k, v, o} of every layer and adapter a,
 *     y = W_P x + scale * B_P[a] (A_P[a] x),
 * the adapter being chosen per sequence (sd_ctx_set_adapters), so that sequences routed to
 * different drafts run as ONE batch of the base model.  a_P / b_P are HOST arrays of n_layers
 * HOST pointers to [n_adapters][rank][d_model] / [n_adapters][d_model][rank] in the model's
 * dtype (fp32 values or bf16 bit patterns); a NULL array leaves that projection unadapted.
 * The factors are copied (as fp32) into device memory the model owns; the low-rank products
 * are computed in fp32.  1 <= rank <= 16.  Replaces adapters set before; n_adapters = 0
 * removes them.  Synchronises. */
typedef struct {
    int32_t n_adapters, rank;
    float scale;
    const void *const *a_q, *const *b_q, *const *a_k, *const *b_k, *const *a_v, *const *b_v, *const *a_o, *const *b_o;
} sd_lora_weights;
int sd_model_set_lora(sd_model *m, const sd_lora_weights *w);

/* A context of `batch` sequences; caps (host, int32[batch]) is each sequence's
 * capacity in tokens (prompt + everything generated + gamma + 1 slack).  Allocates
 * the token buffers.  Synchronises. */
int sd_ctx_create(int32_t batch, const int32_t *caps, sd_ctx **out);
int sd_ctx_free(sd_ctx *c);

/* Allocate model m's KV cache for every sequence of the context: per layer and head,
 * the tokens of all sequences concatenated at their capacity offsets, K and V each in
 * 32-token tiles stored in the order the attention kernels' matrix-core operands read
 * them (V transposed within a tile).  The layout is internal: caches are filled by the
 * forward passes, or by sd_ctx_set_kv from plain [token][head][head_dim] rows.  At most
 * 8 models per context.  Synchronises. */
int sd_ctx_attach(sd_ctx *c, sd_model *m);

/* Replace the tokens of sequences seq_ids (HOST int32[n_seq], or NULL) with the
 * concatenation in tokens (host), lens (host int32[n_seq], each >= 1), and reset
 * every attached model's cache length for them to 0.  Synchronises. */
int sd_ctx_set_tokens(sd_ctx *c, const int32_t *tokens, const int32_t *lens, const int32_t *seq_ids,
                      int32_t n_seq);

/* Adapter of every sequence of the context for model m (attached): adapter_ids is a HOST
 * int32[B] with values in [-1, n_adapters), -1 = the base weights alone (the default).
 * Cache rows already written keep the values they were computed with.  Synchronises. */
int sd_ctx_set_adapters(sd_ctx *c, sd_model *m, const int32_t *adapter_ids);

/* Feed model m with every token of the selected sequences that its cache does
 * not cover yet, except the pending last one (the step before the hot path).  Each
 * forward takes as many 16-token groups per sequence as the model's max_rows allows
 * (max_rows / (16 * n_seq), at least one), so a larger max_rows means fewer passes
 * over the weights; a power of two of at least 1024 lets the blocks of every
 * projection cover the 256 compute units in whole rounds (8192 tokens of a 7B-shape
 * model: 230 ms at 1024 rows against 289 ms at 576).  max_new (host) is the largest number of tokens any selected
 * sequence still has to feed; it fixes the number of forwards.  Enqueues on stream. */
int sd_prefill(sd_model *m, sd_ctx *c, const int32_t *seq_ids /*dev*/, int32_t n_seq, int32_t max_new,
               void *stream);

/* Draft phase (Section 1, Figure 1a).  For each selected sequence: feed the
 * catch-up rows (tokens the draft's cache lacks, at most 2 once prefilled), then
 * decode gamma candidates autoregressively.  temperature > 0: candidate i is
 * drawn by inverse CDF in index order from q_i = softmax(logits_i / T) with
 * uniforms[j][i]; q[j][i][:] receives the full fp32 distribution.  temperature
 * == 0 (greedy): candidate = argmax (ties to the lowest id); q and uniforms are
 * not touched and may be NULL.  The last candidate is not fed to the draft.
 *   uniforms dev fp32 [n_seq][gamma], cand dev int32 [n_seq][gamma],
 *   q dev fp32 [n_seq][gamma][vocab].  1 <= gamma <= 15.
 * The draft's cache must be within two tokens of the sequence (sd_prefill it first): a
 * cache further behind raises the device status flag (SD_ESTATE at the next sd_ctx_sync).
 * sd_draft, sd_verify and sd_commit only enqueue kernels on `stream` (no allocation,
 * copy, memset or host synchronisation; option "profile" off), so they may be
 * captured into a HIP graph and the graph replayed while the sequences grow: results never
 * depend on the host-side length bound of capture time (it only sizes launches; the
 * matrix-core attention kernels read the lengths on the device, the plain one sizes its
 * score buffer from the largest sequence capacity). */
int sd_draft(sd_model *draft, sd_ctx *c, const int32_t *seq_ids /*dev*/, int32_t n_seq, int32_t gamma,
             float temperature, const float *uniforms, int32_t *cand, float *q, void *stream);

/* Verify phase (Section 1, Figure 1b; rule of Section 3.1).  For each selected
 * sequence the target scores the gamma+1 rows (pending token, cand_1..cand_gamma)
 * in one forward pass against its cache, with a causal mask over the new rows.
 * With p_i = softmax(logits_i / T): candidate i is accepted iff
 * uniforms[j][i] < p_i(cand_i) / q_i(cand_i), scanning i = 1..gamma and stopping
 * at the first rejection; n_accepted counts the accepted ones.  The next token is
 * drawn with uniforms[j][gamma] by inverse CDF from norm(max(0, p - q)) of the
 * rejected position, or from p_{gamma+1} if all were accepted.  temperature == 0:
 * accept iff cand_i == argmax logits_i, next = argmax of the first unmatched row.
 * gamma == 0 is one plain autoregressive step of the target.
 * commit != 0 also performs sd_commit's update inside the same kernel.
 *   cand dev int32 [n_seq][gamma]; q dev fp32 [n_seq][gamma][vocab] (NULL if
 *   greedy); uniforms dev fp32 [n_seq][gamma+1] (NULL if greedy);
 *   n_accepted, next_token dev int32 [n_seq].  0 <= gamma <= 15. */
int sd_verify(sd_model *target, sd_ctx *c, const int32_t *seq_ids /*dev*/, int32_t n_seq, int32_t gamma,
              float temperature, const int32_t *cand, const float *q, const float *uniforms,
              int32_t *n_accepted, int32_t *next_token, int32_t commit, void *stream);

/* The acceptance rule alone (Section 3.1; the last stage of sd_verify) on logits the caller holds:
 * the same softmax / accept scan / residual / resample kernels, no model, no context, no commit.
 *   logits dev fp32 [n_seq][gamma+1][vocab] (16-byte aligned); cand, q, uniforms, n_accepted,
 *   next_token as for sd_verify (q 16-byte aligned);
 *   workspace dev fp32 [3 * n_seq * (gamma+1)]: per-row (max, sum of exponentials, argmax) passed
 *   from the first kernel to the second; contents on entry do not matter.
 * vocab a multiple of 4 in [4, 262144]; 0 <= gamma <= 15.  Only enqueues kernels on `stream`. */
int sd_accept(const float *logits, int32_t n_seq, int32_t gamma, int32_t vocab, float temperature,
              const int32_t *cand, const float *q, const float *uniforms, int32_t *n_accepted,
              int32_t *next_token, float *workspace, void *stream);

/* sd_accept for callers that cannot allocate or carry a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments and results, but the
 * per-row statistics live in a fixed device array inside the library (48 KiB per GPU, held until
 * the process ends) instead of a caller's workspace.  Calls no allocating routine; the first call
 * on a device only looks up that device's address of the array.
 * n_seq * (gamma + 1) <= 4096, else SD_ECAP (nothing is enqueued).  All calls on one GPU share the
 * array: two calls whose kernels may overlap on that GPU (different streams) race - serialise them. */
int sd_accept_static(const float *logits, int32_t n_seq, int32_t gamma, int32_t vocab, float temperature,
                     const int32_t *cand, const float *q, const float *uniforms, int32_t *n_accepted,
                     int32_t *next_token, void *stream);

/* Commit / KV rollback: append cand[0..n_accepted) and next_token to each selected
 * sequence, then set every attached model's cache length to
 * min(its length, new token count - 1).  No cache data moves: rows of rejected
 * candidates are dead and get overwritten by the next append. */
int sd_commit(sd_ctx *c, const int32_t *seq_ids /*dev*/, int32_t n_seq, int32_t gamma, const int32_t *cand,
              const int32_t *n_accepted, const int32_t *next_token, void *stream);

/* Routing (Sections 2.1, 2.4): draft_id[i] = argmax_k (W[k] . prompt_emb[i] + b[k]),
 * ties to the lowest id.  All pointers dev; b may be NULL.
 *   W fp32 [n_drafts][emb_dim], prompt_emb fp32 [n][emb_dim], draft_id int32 [n]. */
int sd_route(const float *W, const float *b, int32_t n_drafts, int32_t emb_dim, const float *prompt_emb,
             int32_t n, int32_t *draft_id, void *stream);

/* ---- prompt classifier (Sections 2.4, 3.3.3): the second routing backend ----
 *
 * The classifier the paper describes: an embedding, one selective state-space ("Mamba")
 * sequence layer, average pooling over the prompt's tokens and a linear layer, whose arg
 * max names the draft.  For an embedded prompt u [L][d_model]:
 *   (x, z)  = u W_in                               halves of width d_inner
 *   x_t     = SiLU(b_conv + sum_j w_conv[:, j] x_{t-(d_conv-1)+j})   causal, zero history
 *   (r,B,C) = x_t W_x                              widths dt_rank, d_state, d_state
 *   Delta_t = softplus(r W_dt + b_dt)
 *   h_t     = exp(Delta_t A) h_{t-1} + Delta_t B_t x_t,   A = -exp(a_log),  h_{-1} = 0
 *   y_t     = (C_t . h_t + D x_t) SiLU(z_t),   o_t = y_t W_out
 *   logits  = W_fc mean_t(o_t) + b_fc
 * All arithmetic is fp32.  No normalisation and no residual surround the layer.  u W_in depends on
 * the token id alone, so the library multiplies the embedding and W_in out once, at creation,
 * into a [vocab][2 d_inner] table (device memory: 8 vocab d_inner bytes). */
typedef struct sd_classifier sd_classifier; /* opaque: the classifier's weights on one device */

typedef struct sd_classifier_shape {
    int32_t vocab;     /* >= 1 */
    int32_t d_model;   /* 1..512 */
    int32_t d_inner;   /* a multiple of 64 in 64..512; d_inner * (dt_rank + 2 d_state + 16) + d_model floats must fit
                          64 KB of LDS (else SD_EINVAL) */
    int32_t d_state;   /* 1..16 */
    int32_t dt_rank;   /* 1..16 */
    int32_t d_conv;    /* 1..4 */
    int32_t n_classes; /* 1..64 */
} sd_classifier_shape;

/* Host pointers, fp32, read before sd_classifier_create returns (the library keeps its own
 * device copy).  Matrices are [in features][out features] unless stated. */
typedef struct sd_classifier_weights {
    const float *emb;    /* [vocab][d_model] */
    const float *w_in;   /* [d_model][2 d_inner]: x columns first, then z */
    const float *conv_w; /* [d_inner][d_conv]: the last tap meets the current token */
    const float *conv_b; /* [d_inner] */
    const float *w_x;    /* [d_inner][dt_rank + 2 d_state]: r, then B, then C */
    const float *w_dt;   /* [dt_rank][d_inner] */
    const float *b_dt;   /* [d_inner] */
    const float *a_log;  /* [d_inner][d_state] */
    const float *d;      /* [d_inner] */
    const float *w_out;  /* [d_inner][d_model] */
    const float *w_fc;   /* [n_classes][d_model] */
    const float *b_fc;   /* [n_classes] */
} sd_classifier_weights;

/* Builds a classifier on the current device.  SD_EINVAL for a null pointer or a shape outside
 * the ranges above, SD_EHIP if the device copy fails; *out is NULL on failure. */
int sd_classifier_create(const sd_classifier_shape *shape, const sd_classifier_weights *w, sd_classifier **out);
void sd_classifier_destroy(sd_classifier *c); /* NULL is a no-op; synchronise the streams that use it first */

/* Routing by the classifier: draft_id[i] = arg max of prompt i's logits, ties to the lowest id.
 *   tokens  dev int32 [n][max_len]: prompt i's ids in its first lens[i] slots (the rest is ignored)
 *   lens    dev int32 [n], clamped to [0, max_len]; an empty prompt pools to zero (logits = b_fc)
 *   logits  dev fp32 [n][n_classes], or NULL if not wanted
 *   draft_id dev int32 [n]; -1 for a prompt holding an id outside [0, vocab) (such a token is
 *            embedded as zero and the prompt's logits are still written)
 * Only enqueues one kernel on `stream` (one workgroup per prompt); never synchronises or allocates.
 * SD_EINVAL for a null pointer, n or max_len below 1, or a current device other than the classifier's. */
int sd_route_classifier(const sd_classifier *c, const int32_t *tokens, const int32_t *lens, int32_t n,
                        int32_t max_len, float *logits, int32_t *draft_id, void *stream);

/* ---- candidate-count policy (host only: no GPU call, plain host pointers) ---- */

/* Equation 1 (Section 1): the expected speed-up over autoregressive decoding with gamma
 * candidates per step, per-token acceptance probability alpha in [0, 1] and draft/target
 * cost ratio c >= 0:  (1 - alpha^(gamma+1)) / ((1 - alpha) (gamma c + 1)), whose numerator
 * is gamma + 1 at alpha = 1.  Returns a NaN for arguments outside those ranges. */
double sd_eq1_speedup(double alpha, int32_t gamma, double c);
/* The gamma in [0, gamma_max] (gamma_max <= 15) that maximises Equation 1, the smallest
 * one on ties; 0 means plain autoregressive decoding.  *speedup (may be NULL) receives the
 * maximum.  Returns -1 (and sets the error string) for arguments out of range. */
int32_t sd_choose_gamma(double alpha, double c, int32_t gamma_max, double *speedup);
/* Running estimate of Equation 1's alpha from the n_accepted values of n_steps verify calls
 * at `gamma` candidates: accepted candidates over examined ones, a step that rejects at
 * position k having examined k + 1 (Equation 2's rate counts all gamma instead).  Returns
 * a NaN when nothing was examined or a value is outside [0, gamma]. */
double sd_alpha_hat(const int32_t *n_accepted /*host*/, int32_t n_steps, int32_t gamma);

/* ---- candidate counts per sequence: Equation 1 inside the loop ----
 *
 * A context keeps, per sequence, the accepted and the examined candidates so far (updated on the device by every
 * commit; reset by sd_ctx_set_tokens): their ratio is the running estimate of Equation 1's alpha.  It can also
 * carry a candidate count per sequence.  While it does, sd_draft / sd_verify / sd_commit called with `gamma` row
 * slots let sequence b draft, verify and commit g_b = min(count_b, gamma) candidates: the draft leaves
 * cand[j][g_b..] and q[j][g_b..] untouched, the verify feeds g_b + 1 rows of it, tests uniforms[j][0..g_b) and
 * draws the next token with uniforms[j][g_b]; g_b = 0 is a plain autoregressive step of that sequence.  Array
 * strides stay those of `gamma`.  The batch still moves in lockstep: no host synchronisation is added. */

/* Counts given by the host: gammas host int32[B], each in [0, 15]; NULL switches per-sequence counts off (the
 * default).  Synchronises. */
int sd_policy_set(sd_ctx *c, const int32_t *gammas);
/* Counts chosen on the device for the selected sequences (seq_ids dev, or NULL): for each, alpha = accepted /
 * examined (alpha0 while nothing was examined) and the count in [0, gamma_max] that maximises Equation 1 with
 * cost ratio c_ratio, the smallest on ties - the same arithmetic, operation by operation, as sd_choose_gamma.
 * Switches per-sequence counts on (sequences never chosen for keep gamma_max).  gammas_out: dev int32[n_seq], or
 * NULL.  Enqueues one kernel on `stream` (the first call after sd_policy_set(NULL) also synchronises). */
int sd_policy_choose(sd_ctx *c, const int32_t *seq_ids /*dev*/, int32_t n_seq, double c_ratio, int32_t gamma_max,
                     double alpha0, int32_t *gammas_out, void *stream);
/* Host copies (int32[B] each, any may be NULL) of the counts and of the accepted / examined totals.  Returns 1 if
 * per-sequence counts are on, 0 if off, a negative sd_status on failure.  Synchronises. */
int sd_policy_read(sd_ctx *c, int32_t *gammas, int32_t *accepted, int32_t *examined);

/* ---- inspection and test hooks (synchronising; not on the hot path) ---- */

/* Copy token counts (and model m's cache lengths, if m and kv_len are non-NULL) to
 * host arrays int32[batch]; refresh the host-side length bounds used for launch
 * sizing; return SD_ESTATE if a kernel flagged an inconsistency (row beyond
 * capacity, verify on a sequence whose cache is not at n-1). */
int sd_ctx_sync(sd_ctx *c, sd_model *m, int32_t *n_tokens, int32_t *kv_len);
/* Copy up to max_tokens tokens of sequence seq to host; *n_out = its length. */
int sd_ctx_get_tokens(sd_ctx *c, int32_t seq, int32_t *out, int32_t max_tokens, int32_t *n_out);
/* Load synthetic cache rows for one layer and sequence: k, v arrays
 * [len][n_heads][head_dim] in the model's dtype, in HOST or DEVICE memory; sets
 * that model's cache length for the sequence to len. */
int sd_ctx_set_kv(sd_ctx *c, sd_model *m, int32_t layer, int32_t seq, const void *k, const void *v, int32_t len);
/* KV rollback by hand: set model m's cache length for sequence seq to
 * min(current, len).  Rows beyond stay in memory and are overwritten later. */
int sd_ctx_truncate(sd_ctx *c, sd_model *m, int32_t seq, int32_t len);
/* Copy the fp32 logits [rows][vocab] of model m's last forward into out (dev,
 * room for max_rows rows); *rows = rows copied. */
int sd_last_logits(sd_model *m, float *out, int32_t max_rows, int32_t *rows);
/* Copy one activation buffer of model m's last forward to out (HOST, fp32): name is
 * "x" (residual [rows][d_model]), "qkv" ([rows][3*d_model]), "q", "o", "a"
 * ([rows][d_model]) or "act" ([rows][d_ffn]); "seq_order" / "seq_len" give, for the
 * first `rows` sequences of the last forward, the order attention blocks start in
 * (longest first) and the cache length after that forward.  Synchronises.  Buffers a
 * fused kernel skipped hold older data: "qkv" and "q" whenever attention consumes the
 * QKV GEMM's partial sums directly, "o" when a small model's attention blocks apply the
 * output projection themselves (option "force_generic" selects the unfused kernels). */
int sd_debug_read(sd_model *m, const char *name, float *out, int32_t rows);
/* Host-only (no GPU call): element offset that the library's internal layouts assign.
 * kind 0: tiled bf16 weight [N][K], a = row n, b = column k, c = K  (16-row x 128-column
 *         tiles in MFMA operand order, see sd_load_model);
 * kind 1: step-major activation plane, a = row m, b = column k, c = K, d = rows of the
 *         forward;
 * kind 2: value cache of one head, a = token row t, b = dimension, c = head_dim
 *         (transposed 32-token tiles);
 * kind 3: key cache of one head, same arguments (32-token tiles in MFMA operand order).
 * Returns -1 for an unknown kind or arguments outside the layout's domain. */
int64_t sd_debug_layout_index(int32_t kind, int64_t a, int64_t b, int64_t c, int64_t d);
/* Host-only (no GPU call): the launch plan of a bf16 GEMM with more than 32 rows (the row-blocked kernel).
 * mode 0 = plain projection, 2 = gate/up pair with the SwiGLU epilogue (n = output columns);
 * n_per_seg = output columns per weight segment (n for one matrix, n / 3 for q | k | v).
 * plan[0] = weight rows per block, [1] = rows per block, [2] = column tiles, [3] = row blocks,
 * [4] = K splits, [5] = blocks on the busiest of the 8 dies (column tile t runs on die t mod 8).
 * Returns 0, or SD_EINVAL when the kernel does not take the shape. */
int sd_debug_gemm_plan(int32_t mode, int32_t m, int32_t n, int32_t k, int32_t n_per_seg, int32_t plan[6]);
/* Measurement helper: one kernel that only reads `bytes` bytes (16-byte aligned, dev) once with 16-byte loads,
 * the practical ceiling that the weight-streaming kernels are compared with.  scratch_word: dev uint32, may be
 * written.  Only enqueues on `stream`. */
int sd_debug_stream_read(const void *buf, size_t bytes, uint32_t *scratch_word, void *stream);
/* option "force_generic" = 1 routes every op through the simple reference kernels
 * (2: attention only; 4: only the draft sampler - one block reads the whole logits row
 * instead of starting from the softmax partials the LM head leaves per 32 columns; 8: only
 * the output projection of small models - a GEMM launch of its own instead of a last step of
 * the attention blocks; 0: off).
 * option "profile" = 1 starts bracketing every kernel launch of the forward with HIP
 * events on its stream (a measurement mode: it adds event overhead), 0 stops.
 * option "gemm_splits" = mode*100 + s forces s K splits (1..8; 0 = automatic) for
 * the bf16 GEMMs of mode 0 (plain / residual) or 2 (SwiGLU, ignored): a tuning knob.
 * option "gemm_tile_cols" = 128, 192 or 256 forces the block width (in weight rows) of the
 * row-blocked GEMM for more than 64 rows where the shape allows it (0 = automatic).
 * option "norm_fold": with at most 32 rows in a forward, the add + RMSNorm launches of a
 * layer can be split between the projection before them (adds the residual, applies the gains,
 * leaves per-block sums of squares) and the GEMM after them (scales its sums by 1 / rms); the
 * operand is then rounded to its two bf16 terms before the division by rms instead of after.
 * 0 or 1 = wherever the shapes allow (bf16, no adapters loaded, widths multiples of 128: the
 * default), 2 = never.
 * option "rope_group": on the split attention path (prefill, long contexts) RoPE + cache append of a bf16 model
 * runs one block per (head, group of up to 16 consecutive rows) with 16-byte stores (1, the default) or one block
 * per row (0); both give the same bits.
 * option "prefill_attn": 1 (the default) lets four 16-row groups of a prompt share every K / V tile they
 * read in a prefill forward (one block per four groups and head, tiles staged in LDS); 0 gives every group
 * blocks of its own (the split kernel of the decode path).
 * option "attn_waves" = 4 or 8 forces the block shape of the fused attention kernel
 * (0 = automatic: 4-wave blocks when (sequence, head) pairs oversubscribe the chip and
 * contexts are short).
 * option "stream_read_nt" = 0 makes sd_debug_stream_read a grid-strided read with ordinary loads;
 * 1 (the default) gives every block one contiguous range and reads it with the nontemporal hint,
 * the fastest pattern measured on this part; adding 2 to either turns on a checking mode in which the XOR
 * of every 32-bit word read is folded into *scratch_word (which the caller zeroes), so that a test can
 * tell whether every vector was read exactly once.
 * Unknown names and out-of-range values return SD_EINVAL. */
int sd_set_option(const char *name, int32_t value);
/* Per-kernel-class totals gathered under option "profile": idx = 0,1,.. until
 * SD_EINVAL; *name is a static string, *count launches, *total_ms their summed
 * event-to-event duration.  Synchronises on the recorded events. */
int sd_profile_read(int32_t idx, const char **name, int32_t *count, float *total_ms);

const char *sd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SD_H */
