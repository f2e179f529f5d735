/*
 * Drives every entry point of oracle/sd_oracle.c on a tiny model so that an
 * -fsanitize=address,undefined build of the oracle can be run without Python
 * (tests/test_oracle_sanitize.py compiles this file together with the oracle).
 * Test infrastructure: checks memory safety and defined behaviour only; the
 * oracle's values are pinned by the Python tests.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int dtype;
    double rope_base, rms_eps;
} orc_config;
typedef struct orc_model orc_model;
typedef struct orc_seq orc_seq;

orc_model *orc_model_new(const orc_config *c, const void *embed, const void *lm_head, const float *final_norm,
                         const void *const *wq, const void *const *wk, const void *const *wv, const void *const *wo,
                         const void *const *wgate, const void *const *wup, const void *const *wdown,
                         const float *const *norm_attn, const float *const *norm_ffn);
int orc_model_set_lora(orc_model *m, int n_adapters, int rank, double scale, const void *const *a_q,
                       const void *const *b_q, const void *const *a_k, const void *const *b_k, const void *const *a_v,
                       const void *const *b_v, const void *const *a_o, const void *const *b_o);
void orc_model_free(orc_model *m);
orc_seq *orc_seq_new(const orc_model *m, int cap);
void orc_seq_free(orc_seq *s);
int orc_seq_len(const orc_seq *s);
int orc_seq_set_adapter(const orc_model *m, orc_seq *s, int adapter);
int orc_seq_truncate(orc_seq *s, int len);
int orc_seq_set_kv(const orc_model *m, orc_seq *s, int layer, const void *k, const void *v, int len);
int orc_forward(const orc_model *m, orc_seq *s, const int32_t *tokens, int n_rows, float *logits, int logits_from);
int orc_draft(const orc_model *m, orc_seq *s, const int32_t *ctx, int n, int gamma, double T, const float *u,
              int32_t *cand, float *q, double *margins);
int orc_verify(const orc_model *m, orc_seq *s, const int32_t *ctx, int n, int gamma, double T, const int32_t *cand,
               const float *q, const float *u, int32_t *n_acc, int32_t *next, float *logits_out, double *margins);
void orc_route(const float *W, const float *b, int n_drafts, int emb, const float *e, int n, int32_t *id);
float orc_round_bf16(float f);

static uint64_t g_state = 0x9e3779b97f4a7c15ull;
static double unif(void)
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(g_state >> 11) / 9007199254740992.0;
}
static float small(void) { return (float)((unif() - 0.5) * 0.2); }

static void *matrix(int dtype, size_t n)
{
    if (dtype == 0) {
        float *p = (float *)malloc(n * sizeof(float));
        for (size_t i = 0; i < n; i++) p[i] = small();
        return p;
    }
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; i++) {
        float f = orc_round_bf16(small());
        uint32_t u;
        memcpy(&u, &f, 4);
        p[i] = (uint16_t)(u >> 16);
    }
    return p;
}

static int run(int dtype)
{
    enum { L = 2, D = 32, H = 2, HD = 16, F = 48, V = 40, G = 3, CAP = 24, NA = 2, RK = 3 };
    orc_config c = {L, D, H, HD, F, V, dtype, 10000.0, 1e-5};
    void *embed = matrix(dtype, (size_t)V * D), *lm = matrix(dtype, (size_t)V * D);
    const void *wq[L], *wk[L], *wv[L], *wo[L], *wg[L], *wu[L], *wd[L];
    const void *la[4][L], *lb[4][L];
    const float *na[L], *nf[L];
    float *fin = (float *)malloc(D * sizeof(float));
    for (int i = 0; i < D; i++) fin[i] = 1.0f + small();
    for (int l = 0; l < L; l++) {
        wq[l] = matrix(dtype, D * D), wk[l] = matrix(dtype, D * D), wv[l] = matrix(dtype, D * D);
        wo[l] = matrix(dtype, D * D), wg[l] = matrix(dtype, F * D), wu[l] = matrix(dtype, F * D);
        wd[l] = matrix(dtype, D * F);
        float *a = (float *)malloc(D * sizeof(float)), *b = (float *)malloc(D * sizeof(float));
        for (int i = 0; i < D; i++) a[i] = 1.0f + small(), b[i] = 1.0f + small();
        na[l] = a, nf[l] = b;
        for (int p = 0; p < 4; p++) la[p][l] = matrix(dtype, NA * RK * D), lb[p][l] = matrix(dtype, NA * D * RK);
    }
    orc_model *m = orc_model_new(&c, embed, lm, fin, wq, wk, wv, wo, wg, wu, wd, na, nf);
    if (orc_model_set_lora(m, NA, RK, 0.5, la[0], lb[0], la[1], lb[1], NULL, NULL, la[3], lb[3]) != 0) return 1;
    orc_seq *s = orc_seq_new(m, CAP), *dseq = orc_seq_new(m, CAP);
    if (orc_seq_set_adapter(m, dseq, 1) != 0 || orc_seq_set_adapter(m, dseq, NA) == 0) return 2;
    int32_t ctx[CAP] = {3, 1, 4, 1, 5, 9, 2, 6};
    int n = 8;
    float *logits = (float *)malloc(sizeof(float) * (G + 1) * V);
    /* prefill all but the pending token, row by row and in one piece */
    if (orc_forward(m, s, ctx, n - 1, NULL, n - 1) != 0) return 3;
    if (orc_forward(m, dseq, ctx, 3, logits, 2) != 0 || orc_forward(m, dseq, ctx + 3, n - 4, NULL, n - 4) != 0) return 4;
    for (int step = 0; step < 3; step++) {
        float u[G + 1], q[G * V];
        int32_t cand[G], n_acc = -1, next = -1;
        double mg[G + 1];
        for (int i = 0; i <= G; i++) u[i] = (float)unif();
        const double T = step == 2 ? 0.0 : 0.9;
        if (orc_draft(m, dseq, ctx, n, G, T, u, cand, q, mg) != 0) return 5;
        if (orc_verify(m, s, ctx, n, G, T, cand, q, u, &n_acc, &next, logits, mg) != 0) return 6;
        if (n_acc < 0 || n_acc > G || next < 0 || next >= V) return 7;
        for (int i = 0; i < n_acc; i++) ctx[n++] = cand[i];
        ctx[n++] = next;
        if (orc_seq_truncate(s, n - 1) != 0) return 8;
        if (orc_seq_truncate(dseq, orc_seq_len(dseq) < n - 1 ? orc_seq_len(dseq) : n - 1) != 0) return 9;
    }
    int32_t n_acc, next;
    float u1[1] = {0.25f};
    if (orc_verify(m, s, ctx, n, 0, 1.0, NULL, NULL, u1, &n_acc, &next, NULL, NULL) != 0) return 10; /* gamma = 0 */
    /* synthetic cache rows, full capacity; overflow and bad ids are refused, not executed */
    void *k = matrix(dtype, (size_t)CAP * D), *v = matrix(dtype, (size_t)CAP * D);
    for (int l = 0; l < L; l++)
        if (orc_seq_set_kv(m, s, l, k, v, CAP - 1) != 0) return 11;
    if (orc_seq_set_kv(m, s, 0, k, v, CAP + 1) == 0 || orc_seq_set_kv(m, s, L, k, v, 1) == 0) return 12;
    int32_t one[2] = {7, V};
    if (orc_forward(m, s, one, 1, logits, 0) != 0) return 13;  /* fills the last row */
    if (orc_forward(m, s, one, 1, logits, 0) == 0) return 14;  /* full */
    if (orc_seq_truncate(s, 2) != 0 || orc_forward(m, s, one + 1, 1, logits, 0) == 0) return 15; /* id == vocab */
    float W[4 * 6], e[3 * 6];
    int32_t id[3];
    for (int i = 0; i < 24; i++) W[i] = small();
    for (int i = 0; i < 18; i++) e[i] = small();
    orc_route(W, NULL, 4, 6, e, 3, id);
    orc_seq_free(s);
    orc_seq_free(dseq);
    orc_model_free(m);
    free(k); free(v); free(logits); free(fin); free(embed); free(lm);
    for (int l = 0; l < L; l++) {
        free((void *)wq[l]); free((void *)wk[l]); free((void *)wv[l]); free((void *)wo[l]);
        free((void *)wg[l]); free((void *)wu[l]); free((void *)wd[l]); free((void *)na[l]); free((void *)nf[l]);
        for (int p = 0; p < 4; p++) free((void *)la[p][l]), free((void *)lb[p][l]);
    }
    return 0;
}

int main(void)
{
    for (int dtype = 0; dtype < 2; dtype++) {
        int rc = run(dtype);
        if (rc) {
            printf("driver step %d failed (dtype %d)\n", rc, dtype);
            return 1;
        }
    }
    printf("sanitize driver ok\n");
    return 0;
}
