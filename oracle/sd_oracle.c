/*
 * CPU oracle for the draft-then-verify step of speculative decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * statement of what the HIP library must compute.  It shares no code, header,
 * table or constant with the HIP path; only tests, the smoke check and the
 * bench's cpu_baseline leg may call it.
 *
 * What it follows (paper = arXiv 2505.08600):
 *   - Section 1 / Figure 1: a draft model decodes gamma candidate tokens
 *     autoregressively (a), the target model scores them in one parallel pass (b).
 *   - Section 3.1 "Parameter Settings": verification is the non-deterministic
 *     (speculative sampling) rule of the work the paper cites for Equation 1:
 *     accept candidate c with probability min(1, p(c)/q(c)); on the first
 *     rejection resample from norm(max(0, p - q)); if all gamma are accepted
 *     draw one more token from the target's next distribution.  Greedy decoding
 *     is the T -> 0 limit: accept iff c equals the target's argmax.
 *   - Section 3.1 "Models": LLaMA-family target and draft => pre-norm decoder
 *     block with RMSNorm, rotary position embedding (rotate-half pairing),
 *     multi-head causal attention, SwiGLU feed-forward, untied LM head, no biases.
 *
 * Numeric contract (the paper states no precision; this is this build's reading):
 *   fp32 models: weights, KV cache and GEMM inputs are fp32 values.
 *   bf16 models: weights, embedding table and KV cache are bf16 values (round to
 *   nearest even from fp32).  Every activation that enters a contraction (normed
 *   hidden, rotated q, attention output, SwiGLU product) is the sum of two bf16
 *   terms, hi = bf16(x), lo = bf16(x - hi): about 16 mantissa bits, so that two
 *   implementations that add in different orders do not drift apart through
 *   differing roundings (with single bf16 activations the drift between two
 *   correct implementations was measured at 2.8e-2 of the logit range over 32
 *   layers - outside the 2e-2 tolerance and far outside a 1e-3 decision band).
 *   Everything else is wider.
 *   Between those rounding points this oracle computes in fp64.  Logits leave as
 *   fp32 and are never rounded to bf16.  Decisions (accept test, argmax) are taken
 *   on fp32 logits / probabilities, the precision the kernels decide in.
 *
 * Pins (tests/test_oracle_*.py): an independent LLaMA implementation from a
 * third-party library on the same weights, row-by-row vs multi-row forward,
 * RoPE relative-position property, uniform-attention closed form, greedy
 * speculative decoding == plain target decoding, exact enumeration of the
 * emitted-token law on tiny vocabularies, the closed form of Equation 1's
 * numerator for the expected tokens per step, and special cases (draft ==
 * target, impossible candidate, gamma == 0).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_FP32 0
#define ORC_BF16 1
#define ORC_INF 1e30

typedef struct {
    int n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int dtype;
    double rope_base, rms_eps;
} orc_config;

/* Low-rank adapters on the attention projections (Section 2.3: the heterogeneous drafts are LoRA
 * fine-tunes of one base model).  For projection P in {q, k, v, o} of layer l and adapter a:
 *   y = W x + scale * B[a] (A[a] x),  A[a]: [rank][in], B[a]: [out][rank],
 * stored per layer as [n_adapters][rank][in] and [n_adapters][out][rank] in the model's dtype.
 * A NULL pointer array means that projection is not adapted. */
typedef struct {
    int n_adapters, rank;
    double scale;
    const void **a[4], **b[4]; /* q, k, v, o */
} orc_lora;

typedef struct {
    orc_config c;
    const void *embed, *lm_head;
    const float *final_norm;
    const void **wq, **wk, **wv, **wo, **wgate, **wup, **wdown;
    const float **norm_attn, **norm_ffn;
    orc_lora lora; /* n_adapters == 0: none */
} orc_model;

/* One sequence's KV cache for one model: k, v are [n_layers][cap][n_heads*head_dim],
 * holding values already rounded to the model's storage type.  adapter: the sequence's
 * low-rank adapter for this model (-1: the base weights alone). */
typedef struct {
    int cap, len;
    float *k, *v;
    int adapter;
} orc_seq;

/* ---------- rounding points ---------- */

static float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32 -> nearest bf16 (ties to even), returned as the fp32 value it denotes. */
static float round_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f; /* NaN stays NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return f;
}

/* Exported for the rounding pin. */
float orc_round_bf16(float f) { return round_to_bf16(f); }

/* Value as stored in the KV cache of a model of this dtype. */
static double round_storage(double x, int dtype)
{
    float f = (float)x;
    return dtype == ORC_BF16 ? (double)round_to_bf16(f) : (double)f;
}

/* Value of a GEMM / attention input activation.  fp32 models: the fp32 value.
 * bf16 models: the sum of two bf16 terms, hi = bf16(x) and lo = bf16(x - hi),
 * i.e. about 16 mantissa bits, each term a bf16 operand of the matrix cores. */
static double round_act(double x, int dtype)
{
    float f = (float)x;
    if (dtype != ORC_BF16) return (double)f;
    float hi = round_to_bf16(f);
    float lo = round_to_bf16(f - hi);
    return (double)hi + (double)lo;
}

static double weight_at(const void *w, int dtype, size_t i)
{
    return dtype == ORC_BF16 ? (double)bf16_bits_to_float(((const uint16_t *)w)[i])
                             : (double)((const float *)w)[i];
}

/* ---------- exported building blocks (also called by the pins) ---------- */

/* RMSNorm: out_i = x_i / sqrt(mean(x^2) + eps) * g_i. */
void orc_rmsnorm(const double *x, const float *g, int d, double eps, double *out)
{
    double ss = 0.0;
    for (int i = 0; i < d; i++) ss += x[i] * x[i];
    double inv = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; i++) out[i] = x[i] * inv * (double)g[i];
}

/* Rotary embedding of one head vector at position pos, rotate-half pairing:
 * element i pairs with i + hd/2, angle pos * base^(-2i/hd). */
void orc_rope(double *x, int hd, int pos, double base)
{
    int half = hd / 2;
    for (int i = 0; i < half; i++) {
        double theta = pow(base, -2.0 * i / hd);
        double c = cos(pos * theta), s = sin(pos * theta);
        double a = x[i], b = x[i + half];
        x[i] = a * c - b * s;
        x[i + half] = b * c + a * s;
    }
}

/* y[n] = sum_k W[n][k] * a[k], W row-major [N][K] in the model's dtype. */
static void matvec(const void *W, int dtype, int N, int K, const double *a, double *y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; n++) {
        double acc = 0.0;
        if (dtype == ORC_BF16) {
            const uint16_t *w = (const uint16_t *)W + (size_t)n * K;
            for (int k = 0; k < K; k++) acc += (double)bf16_bits_to_float(w[k]) * a[k];
        } else {
            const float *w = (const float *)W + (size_t)n * K;
            for (int k = 0; k < K; k++) acc += (double)w[k] * a[k];
        }
        y[n] = acc;
    }
}

/* y[n] += scale * sum_j B[n][j] * (sum_k A[j][k] * x[k]): the low-rank update of one projection,
 * A: [rank][K], B: [N][rank] of the sequence's adapter. */
static void lora_add(const orc_lora *lo, int proj, int layer, int adapter, int dtype, int N, int K, const double *x,
                     double *y)
{
    if (lo->n_adapters == 0 || adapter < 0 || !lo->a[proj] || !lo->b[proj]) return;
    const int r = lo->rank;
    const size_t a0 = (size_t)adapter * r * K, b0 = (size_t)adapter * N * r;
    double t[64];
    for (int j = 0; j < r; j++) {
        double acc = 0.0;
        for (int k = 0; k < K; k++) acc += weight_at(lo->a[proj][layer], dtype, a0 + (size_t)j * K + k) * x[k];
        t[j] = acc;
    }
    for (int n = 0; n < N; n++) {
        double acc = 0.0;
        for (int j = 0; j < r; j++) acc += weight_at(lo->b[proj][layer], dtype, b0 + (size_t)n * r + j) * t[j];
        y[n] += lo->scale * acc;
    }
}

/* Temperature softmax of one fp32 logit row, in fp64; p is stored as fp32. */
void orc_softmax_T(const float *logits, int V, double T, float *p)
{
    double mx = -ORC_INF, z = 0.0;
    for (int i = 0; i < V; i++)
        if (logits[i] > mx) mx = logits[i];
    for (int i = 0; i < V; i++) z += exp(((double)logits[i] - mx) / T);
    for (int i = 0; i < V; i++) p[i] = (float)(exp(((double)logits[i] - mx) / T) / z);
}

/* argmax with ties to the lowest index; *gap = top1 - top2 (in the row's units). */
int orc_argmax(const float *x, int V, double *gap)
{
    int best = 0;
    for (int i = 1; i < V; i++)
        if (x[i] > x[best]) best = i;
    double second = -ORC_INF;
    for (int i = 0; i < V; i++)
        if (i != best && x[i] > second) second = x[i];
    if (gap) *gap = V > 1 ? (double)x[best] - second : ORC_INF;
    return best;
}

/* Inverse-CDF draw in index order from non-negative weights w (need not be
 * normalised): the smallest k with sum_{x<=k} w_x > u * sum_x w_x.  If rounding
 * leaves no such k, the last index with positive weight.  *margin = distance of
 * u from the nearer edge of k's interval, as a fraction of the total mass. */
int orc_sample_cdf(const double *w, int V, double u, double *margin)
{
    double Z = 0.0;
    for (int i = 0; i < V; i++) Z += w[i];
    double target = u * Z, cdf = 0.0;
    int pick = -1, last_pos = 0;
    double lo = 0.0, hi = 0.0;
    for (int i = 0; i < V; i++) {
        if (w[i] > 0.0) last_pos = i;
        double next = cdf + w[i];
        if (pick < 0 && next > target) {
            pick = i;
            lo = cdf;
            hi = next;
        }
        cdf = next;
    }
    if (pick < 0) {
        pick = last_pos;
        if (margin) *margin = 0.0;
        return pick;
    }
    if (margin) { /* an edge is a decision boundary only if mass lies beyond it */
        double a = lo > 0.0 ? (target - lo) / Z : ORC_INF;
        double b = hi < Z ? (hi - target) / Z : ORC_INF;
        *margin = a < b ? a : b;
    }
    return pick;
}

/* ---------- model / sequence handles ---------- */

static const void **copy_ptrs(const void *const *p, int n)
{
    const void **r = (const void **)malloc(sizeof(void *) * (size_t)n);
    memcpy(r, p, sizeof(void *) * (size_t)n);
    return r;
}

orc_model *orc_model_new(const orc_config *c, const void *embed, const void *lm_head, const float *final_norm,
                         const void *const *wq, const void *const *wk, const void *const *wv,
                         const void *const *wo, const void *const *wgate, const void *const *wup,
                         const void *const *wdown, const float *const *norm_attn, const float *const *norm_ffn)
{
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->c = *c;
    m->embed = embed;
    m->lm_head = lm_head;
    m->final_norm = final_norm;
    int L = c->n_layers;
    m->wq = copy_ptrs(wq, L);
    m->wk = copy_ptrs(wk, L);
    m->wv = copy_ptrs(wv, L);
    m->wo = copy_ptrs(wo, L);
    m->wgate = copy_ptrs(wgate, L);
    m->wup = copy_ptrs(wup, L);
    m->wdown = copy_ptrs(wdown, L);
    m->norm_attn = (const float **)copy_ptrs((const void *const *)norm_attn, L);
    m->norm_ffn = (const float **)copy_ptrs((const void *const *)norm_ffn, L);
    return m;
}

/* Attach adapters: a_q .. b_o are [n_layers] pointer arrays (or NULL); rank <= 64. */
int orc_model_set_lora(orc_model *m, int n_adapters, int rank, double scale, const void *const *a_q,
                       const void *const *b_q, const void *const *a_k, const void *const *b_k, const void *const *a_v,
                       const void *const *b_v, const void *const *a_o, const void *const *b_o)
{
    if (n_adapters < 0 || rank < 1 || rank > 64) return -1;
    const void *const *as[4] = {a_q, a_k, a_v, a_o}, *const *bs[4] = {b_q, b_k, b_v, b_o};
    for (int p = 0; p < 4; p++) {
        free(m->lora.a[p]);
        free(m->lora.b[p]);
        m->lora.a[p] = as[p] ? copy_ptrs(as[p], m->c.n_layers) : NULL;
        m->lora.b[p] = bs[p] ? copy_ptrs(bs[p], m->c.n_layers) : NULL;
    }
    m->lora.n_adapters = n_adapters;
    m->lora.rank = rank;
    m->lora.scale = scale;
    return 0;
}

void orc_model_free(orc_model *m)
{
    if (!m) return;
    for (int p = 0; p < 4; p++) {
        free(m->lora.a[p]);
        free(m->lora.b[p]);
    }
    free(m->wq); free(m->wk); free(m->wv); free(m->wo);
    free(m->wgate); free(m->wup); free(m->wdown);
    free(m->norm_attn); free(m->norm_ffn);
    free(m);
}

orc_seq *orc_seq_new(const orc_model *m, int cap)
{
    orc_seq *s = (orc_seq *)calloc(1, sizeof(orc_seq));
    size_t n = (size_t)m->c.n_layers * cap * m->c.n_heads * m->c.head_dim;
    s->cap = cap;
    s->len = 0;
    s->adapter = -1;
    s->k = (float *)calloc(n, sizeof(float));
    s->v = (float *)calloc(n, sizeof(float));
    return s;
}

void orc_seq_free(orc_seq *s)
{
    if (!s) return;
    free(s->k);
    free(s->v);
    free(s);
}

int orc_seq_len(const orc_seq *s) { return s->len; }

/* Choose the sequence's adapter for its model (-1: none).  Cache rows already written keep
 * the values they were computed with. */
int orc_seq_set_adapter(const orc_model *m, orc_seq *s, int adapter)
{
    if (adapter < -1 || adapter >= m->lora.n_adapters) return -1;
    s->adapter = adapter;
    return 0;
}

/* KV rollback: rows at index >= len are dead; nothing moves. */
int orc_seq_truncate(orc_seq *s, int len)
{
    if (len < 0 || len > s->len) return -1;
    s->len = len;
    return 0;
}

/* Load synthetic cache contents for one layer: k, v are [len][n_heads][head_dim]
 * in the model's dtype (fp32 values or bf16 bit patterns).  Sets the length. */
int orc_seq_set_kv(const orc_model *m, orc_seq *s, int layer, const void *k, const void *v, int len)
{
    int HD = m->c.n_heads * m->c.head_dim;
    if (len > s->cap || layer < 0 || layer >= m->c.n_layers) return -1;
    float *kd = s->k + (size_t)layer * s->cap * HD, *vd = s->v + (size_t)layer * s->cap * HD;
    for (size_t i = 0; i < (size_t)len * HD; i++) {
        kd[i] = (float)weight_at(k, m->c.dtype, i);
        vd[i] = (float)weight_at(v, m->c.dtype, i);
    }
    s->len = len;
    return 0;
}

/* ---------- the decoder forward ---------- */

/* Feed n_rows tokens at positions len .. len+n_rows-1, append their K/V, and
 * write fp32 logits for rows >= logits_from into logits[(row-logits_from)][V]
 * (logits may be NULL when logits_from >= n_rows).  Returns 0, or -1 on overflow
 * or a token id outside the vocabulary. */
int orc_forward(const orc_model *m, orc_seq *s, const int32_t *tokens, int n_rows, float *logits, int logits_from)
{
    const orc_config *c = &m->c;
    const int d = c->d_model, H = c->n_heads, hd = c->head_dim, HD = H * hd, F = c->d_ffn, V = c->vocab, dt = c->dtype;
    if (n_rows <= 0) return 0;
    if (s->len + n_rows > s->cap) return -1;
    for (int r = 0; r < n_rows; r++)
        if (tokens[r] < 0 || tokens[r] >= V) return -1;

    double *h = (double *)malloc(sizeof(double) * (size_t)n_rows * d);      /* residual stream */
    double *a = (double *)malloc(sizeof(double) * (size_t)(d > F ? d : F)); /* GEMM input (rounded) */
    double *qb = (double *)malloc(sizeof(double) * (size_t)n_rows * HD);    /* rotated, rounded queries */
    double *tmp = (double *)malloc(sizeof(double) * (size_t)(HD > F ? HD : F));
    double *tmp2 = (double *)malloc(sizeof(double) * (size_t)F);
    double *ob = (double *)malloc(sizeof(double) * (size_t)HD);
    double *y = (double *)malloc(sizeof(double) * (size_t)(d > V ? d : V));
    const double inv_sqrt_hd = 1.0 / sqrt((double)hd);

    for (int r = 0; r < n_rows; r++)
        for (int i = 0; i < d; i++) h[(size_t)r * d + i] = weight_at(m->embed, dt, (size_t)tokens[r] * d + i);

    for (int l = 0; l < c->n_layers; l++) {
        float *Kc = s->k + (size_t)l * s->cap * HD, *Vc = s->v + (size_t)l * s->cap * HD;
        /* projections, rotary embedding, cache append: all rows first */
        for (int r = 0; r < n_rows; r++) {
            int pos = s->len + r;
            orc_rmsnorm(h + (size_t)r * d, m->norm_attn[l], d, c->rms_eps, a);
            for (int i = 0; i < d; i++) a[i] = round_act(a[i], dt);
            matvec(m->wq[l], dt, HD, d, a, tmp);
            lora_add(&m->lora, 0, l, s->adapter, dt, HD, d, a, tmp);
            for (int hh = 0; hh < H; hh++) orc_rope(tmp + hh * hd, hd, pos, c->rope_base);
            for (int i = 0; i < HD; i++) qb[(size_t)r * HD + i] = round_act(tmp[i], dt);
            matvec(m->wk[l], dt, HD, d, a, tmp);
            lora_add(&m->lora, 1, l, s->adapter, dt, HD, d, a, tmp);
            for (int hh = 0; hh < H; hh++) orc_rope(tmp + hh * hd, hd, pos, c->rope_base);
            for (int i = 0; i < HD; i++) Kc[(size_t)pos * HD + i] = (float)round_storage(tmp[i], dt);
            matvec(m->wv[l], dt, HD, d, a, tmp);
            lora_add(&m->lora, 2, l, s->adapter, dt, HD, d, a, tmp);
            for (int i = 0; i < HD; i++) Vc[(size_t)pos * HD + i] = (float)round_storage(tmp[i], dt);
        }
        for (int r = 0; r < n_rows; r++) {
            int pos = s->len + r; /* this row sees cache rows 0..pos (causal over the new rows) */
            /* (heads are independent: they may run on different threads; inside a head nothing changes) */
#pragma omp parallel for schedule(static)
            for (int hh = 0; hh < H; hh++) {
                double *sc = (double *)malloc(sizeof(double) * (size_t)(pos + 1)); /* this head's scores */
                const double *q = qb + (size_t)r * HD + hh * hd;
                double mx = -ORC_INF;
                for (int t = 0; t <= pos; t++) {
                    const float *kt = Kc + (size_t)t * HD + hh * hd;
                    double dot = 0.0;
                    for (int i = 0; i < hd; i++) dot += q[i] * (double)kt[i];
                    sc[t] = dot * inv_sqrt_hd;
                    if (sc[t] > mx) mx = sc[t];
                }
                double z = 0.0;
                for (int t = 0; t <= pos; t++) {
                    sc[t] = exp(sc[t] - mx);
                    z += sc[t];
                }
                for (int i = 0; i < hd; i++) {
                    double acc = 0.0;
                    for (int t = 0; t <= pos; t++) acc += sc[t] * (double)Vc[(size_t)t * HD + hh * hd + i];
                    ob[hh * hd + i] = round_act(acc / z, dt);
                }
                free(sc);
            }
            matvec(m->wo[l], dt, d, HD, ob, y);
            lora_add(&m->lora, 3, l, s->adapter, dt, d, HD, ob, y);
            double *hr = h + (size_t)r * d;
            for (int i = 0; i < d; i++) hr[i] += y[i];
            /* SwiGLU feed-forward */
            orc_rmsnorm(hr, m->norm_ffn[l], d, c->rms_eps, a);
            for (int i = 0; i < d; i++) a[i] = round_act(a[i], dt);
            matvec(m->wgate[l], dt, F, d, a, tmp);
            matvec(m->wup[l], dt, F, d, a, tmp2);
            for (int i = 0; i < F; i++) {
                double g = tmp[i];
                a[i] = round_act(g / (1.0 + exp(-g)) * tmp2[i], dt);
            }
            matvec(m->wdown[l], dt, d, F, a, y);
            for (int i = 0; i < d; i++) hr[i] += y[i];
        }
    }
    for (int r = (logits_from < 0 ? 0 : logits_from); r < n_rows; r++) {
        orc_rmsnorm(h + (size_t)r * d, m->final_norm, d, c->rms_eps, a);
        for (int i = 0; i < d; i++) a[i] = round_act(a[i], dt);
        matvec(m->lm_head, dt, V, d, a, y);
        float *out = logits + (size_t)(r - (logits_from < 0 ? 0 : logits_from)) * V;
        for (int i = 0; i < V; i++) out[i] = (float)y[i];
    }
    s->len += n_rows;
    free(h); free(a); free(qb); free(tmp); free(tmp2); free(ob); free(y);
    return 0;
}

/* Weights the next token is drawn from after n_acc accepted candidates (T > 0):
 * the residual max(0, p - q) of the rejected position, or p itself when every
 * candidate was accepted or the residual is numerically empty. */
void orc_next_weights(int V, int gamma, double T, const float *logits, const float *q, int n_acc, double *w)
{
    float *p = (float *)malloc(sizeof(float) * (size_t)V);
    orc_softmax_T(logits + (size_t)n_acc * V, V, T, p);
    double Z = 0.0;
    if (n_acc < gamma) {
        const float *qj = q + (size_t)n_acc * V;
        for (int x = 0; x < V; x++) {
            double r = (double)p[x] - (double)qj[x];
            w[x] = r > 0.0 ? r : 0.0;
            Z += w[x];
        }
    }
    if (!(Z > 0.0))
        for (int x = 0; x < V; x++) w[x] = (double)p[x];
    free(p);
}

/* How far u lies outside token k's interval of the inverse CDF of w, as a
 * fraction of the total mass (0 when k is the token orc_sample_cdf picks, or u
 * sits exactly on its edge).  Used to decide whether another implementation's
 * pick is within rounding of this one's. */
double orc_cdf_distance(const double *w, int V, double u, int k)
{
    double Z = 0.0, lo = 0.0;
    for (int i = 0; i < V; i++) Z += w[i];
    for (int i = 0; i < k; i++) lo += w[i];
    double hi = lo + w[k], target = u * Z;
    if (target < lo) return (lo - target) / Z;
    if (target > hi) return (target - hi) / Z;
    return 0.0;
}

/* ---------- acceptance rule (Section 3.1; rule restated in the header) ---------- */

/* logits: [(gamma+1)][V] fp32 target logits for rows (pending token, c_1..c_gamma);
 * q: [gamma][V] fp32 draft probabilities (ignored when T == 0); u: gamma accept
 * uniforms then one resample/bonus uniform.  margins[i<gamma] = |u_i - ratio_i|
 * (T > 0) or the target's top1-top2 logit gap (T == 0) for examined candidates,
 * margins[gamma] = margin of the next-token decision; unexamined entries = ORC_INF. */
void orc_accept(int V, int gamma, double T, const float *logits, const float *q, const int32_t *cand,
                const float *u, int32_t *n_acc_out, int32_t *next_out, double *margins)
{
    double dummy[64];
    if (!margins) margins = dummy;
    for (int i = 0; i <= gamma; i++) margins[i] = ORC_INF;
    int n_acc = 0;
    if (T == 0.0) {
        for (int i = 0; i < gamma; i++) {
            int am = orc_argmax(logits + (size_t)i * V, V, &margins[i]);
            if (am != cand[i]) break;
            n_acc++;
        }
        *n_acc_out = n_acc;
        *next_out = orc_argmax(logits + (size_t)n_acc * V, V, &margins[gamma]);
        return;
    }
    float *p = (float *)malloc(sizeof(float) * (size_t)V);
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    for (int i = 0; i < gamma; i++) {
        orc_softmax_T(logits + (size_t)i * V, V, T, p);
        float qc = q[(size_t)i * V + cand[i]];
        if (qc < 1.17549435e-38f) qc = 1.17549435e-38f;
        float ratio = p[cand[i]] / qc; /* decision in fp32, as the kernel takes it */
        margins[i] = fabs((double)u[i] - (double)ratio);
        if (!(u[i] < ratio)) break; /* u in [0,1): min(1, ratio) is implicit */
        n_acc++;
    }
    *n_acc_out = n_acc;
    orc_next_weights(V, gamma, T, logits, q, n_acc, w);
    *next_out = orc_sample_cdf(w, V, (double)u[gamma], &margins[gamma]);
    free(p);
    free(w);
}

/* ---------- the two calls of the hot path ---------- */

/* Draft: ctx[0..n) is the sequence so far, the draft cache covers [0, m) with
 * m <= n-1.  Feeds the catch-up rows x_m..x_{n-1}, draws c_1 from the last row's
 * distribution, then feeds c_{i-1} to draw c_i.  c_gamma is never fed.  On return
 * the cache covers [0, n-1+gamma).  q: [gamma][V] (not written when T == 0).
 * margins[i]: sampling margin (T > 0) or argmax gap (T == 0) of candidate i. */
int orc_draft(const orc_model *m, orc_seq *s, const int32_t *ctx, int n, int gamma, double T, const float *u,
              int32_t *cand, float *q, double *margins)
{
    int V = m->c.vocab;
    if (gamma < 1 || s->len > n - 1 || n < 1) return -1;
    float *logits = (float *)malloc(sizeof(float) * (size_t)V);
    float *prow = (float *)malloc(sizeof(float) * (size_t)V);
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    int rc = 0;
    for (int i = 0; i < gamma && rc == 0; i++) {
        if (i == 0) {
            int rows = n - s->len;
            rc = orc_forward(m, s, ctx + s->len, rows, logits, rows - 1);
        } else {
            rc = orc_forward(m, s, &cand[i - 1], 1, logits, 0);
        }
        if (rc) break;
        double mg = ORC_INF;
        if (T == 0.0) {
            cand[i] = orc_argmax(logits, V, &mg);
        } else {
            orc_softmax_T(logits, V, T, prow);
            memcpy(q + (size_t)i * V, prow, sizeof(float) * (size_t)V);
            for (int x = 0; x < V; x++) w[x] = (double)prow[x];
            cand[i] = orc_sample_cdf(w, V, (double)u[i], &mg);
        }
        if (margins) margins[i] = mg;
    }
    free(logits); free(prow); free(w);
    return rc;
}

/* Verify: the target cache covers [0, n-1); x_{n-1} is pending.  Feeds the
 * gamma+1 rows (x_{n-1}, c_1..c_gamma), applies the acceptance rule.  gamma == 0
 * is one plain autoregressive step of the target.  Leaves the cache covering
 * [0, n+gamma): the caller commits by truncating to n + n_acc.  logits_out may
 * be NULL, else receives [(gamma+1)][V]. */
int orc_verify(const orc_model *m, orc_seq *s, const int32_t *ctx, int n, int gamma, double T,
               const int32_t *cand, const float *q, const float *u, int32_t *n_acc, int32_t *next,
               float *logits_out, double *margins)
{
    int V = m->c.vocab;
    if (gamma < 0 || gamma > 62 || n < 1 || s->len != n - 1) return -1;
    int32_t *rows = (int32_t *)malloc(sizeof(int32_t) * (size_t)(gamma + 1));
    float *logits = (float *)malloc(sizeof(float) * (size_t)(gamma + 1) * V);
    rows[0] = ctx[n - 1];
    for (int i = 0; i < gamma; i++) rows[i + 1] = cand[i];
    int rc = orc_forward(m, s, rows, gamma + 1, logits, 0);
    if (rc == 0) {
        orc_accept(V, gamma, T, logits, q, cand, u, n_acc, next, margins);
        if (logits_out) memcpy(logits_out, logits, sizeof(float) * (size_t)(gamma + 1) * V);
    }
    free(rows);
    free(logits);
    return rc;
}

/* Routing: draft id = argmax_k (W[k] . e + b[k]), ties to the lowest id (Section 2.4:
 * a lightweight classifier picks the draft; here a linear one). */
void orc_route(const float *W, const float *b, int n_drafts, int emb, const float *e, int n, int32_t *id)
{
    for (int i = 0; i < n; i++) {
        int best = 0;
        double bs = -ORC_INF;
        for (int k = 0; k < n_drafts; k++) {
            double sdot = b ? (double)b[k] : 0.0;
            for (int j = 0; j < emb; j++) sdot += (double)W[(size_t)k * emb + j] * (double)e[(size_t)i * emb + j];
            if (sdot > bs) {
                bs = sdot;
                best = k;
            }
        }
        id[i] = best;
    }
}
