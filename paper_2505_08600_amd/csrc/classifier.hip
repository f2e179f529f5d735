// Prompt classifier (Sections 2.4, 3.3.3): embedding -> one selective state-space layer ->
// average pooling over the prompt -> linear layer -> arg max, as the second backend of routing.
//
// One workgroup per prompt, one thread per inner channel.  The recurrence over tokens is
// sequential, so everything a channel needs between tokens (its state row, its convolution
// history, its weights) stays in that thread's registers; only the small per-token projection
// (dt_rank + 2 d_state outputs) crosses threads, through LDS.  The input projection has no
// dependence between tokens and is done for CLS_TC tokens at a time, which divides the reads
// of its weight matrix (from L2) by CLS_TC.  Pooling and the output projection commute (both
// linear), so the channel outputs are averaged first and projected once per prompt.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/sd.h"
#include "sd_internal.h"

#define CLS_TC 8          // tokens per chunk: everything but the state update is done a chunk at a time
#define CLS_MAX_STATE 16
#define CLS_MAX_RANK 16
#define CLS_MAX_CONV 4
#define CLS_MAX_INNER 512
#define CLS_MAX_MODEL 512
#define CLS_MAX_CLASSES 64
#define CLS_LDS_LIMIT (65536 - 64) // dynamic part; the kernel also holds one static word

struct ClsView {
    // table[v] = emb[v] W_in, [vocab][2 d_inner]: the embedding and the input projection are both
    // functions of the token id alone, so the library multiplies them out once at creation.
    const float *table, *conv_w, *conv_b, *w_x, *w_dt, *b_dt, *a_log, *d, *w_out, *w_fc, *b_fc;
    int vocab, d_model, d_inner, d_state, dt_rank, d_conv, n_classes;
};

struct sd_classifier {
    ClsView v;
    void *mem;
    int device;
    size_t lds_bytes;
};

__host__ __device__ static inline size_t cls_align4(size_t n) { return (n + 3) & ~(size_t)3; }

// LDS layout in floats:
//   W_x [d_inner][J] | x [d_inner][CLS_TC] | part [waves][CLS_TC][64] | dbc [CLS_TC][64] | o [d_model + 64]
__host__ __device__ static inline size_t cls_lds_floats(int d_inner, int J, int d_model)
{
    return cls_align4((size_t)d_inner * J) + (size_t)d_inner * CLS_TC + (size_t)(d_inner / 64) * CLS_TC * 64 +
           CLS_TC * 64 + cls_align4((size_t)d_model + CLS_MAX_CLASSES);
}

// table[v][c] = sum_k emb[v][k] W_in[k][c]; one block per vocabulary entry.
__global__ void __launch_bounds__(256)
classifier_table_kernel(const float *__restrict__ emb, const float *__restrict__ w_in, int d_model, int cols,
                        float *__restrict__ table)
{
    __shared__ float e[CLS_MAX_MODEL];
    const size_t v = blockIdx.x;
    for (int k = threadIdx.x; k < d_model; k += blockDim.x) e[k] = emb[v * d_model + k];
    __syncthreads();
    for (int c = threadIdx.x; c < cols; c += blockDim.x) {
        float acc = 0.f;
        for (int k = 0; k < d_model; ++k) acc = fmaf(e[k], w_in[(size_t)k * cols + c], acc);
        table[v * cols + c] = acc;
    }
}

__global__ void __launch_bounds__(CLS_MAX_INNER)
classifier_kernel(ClsView v, const int32_t *__restrict__ tokens, const int32_t *__restrict__ lens, int max_len,
                  float *__restrict__ logits, int32_t *__restrict__ draft_id)
{
    extern __shared__ __align__(16) float lds[];
    const int J = v.dt_rank + 2 * v.d_state;
    const int di = v.d_inner, dm = v.d_model, waves = di >> 6;
    float *s_wx = lds;
    float *s_x = s_wx + cls_align4((size_t)di * J);
    float *s_part = s_x + (size_t)di * CLS_TC;
    float *s_dbc = s_part + (size_t)waves * CLS_TC * 64;
    float *s_o = s_dbc + CLS_TC * 64;
    __shared__ int s_bad;

    const int c = threadIdx.x, lane = c & 63, wave = c >> 6;
    const int i = blockIdx.x;
    int L = lens[i];
    L = L < 0 ? 0 : (L > max_len ? max_len : L);
    const int32_t *tok = tokens + (size_t)i * max_len;

    if (c == 0) s_bad = 0;
    for (int k = c; k < di * J; k += di) s_wx[k] = v.w_x[k];
    // per token, r sits in slots [0, 16), B in [16, 32), C in [32, 48): slots beyond dt_rank / d_state stay
    // zero, so the loops over them below run to the fixed maxima without a branch
    for (int k = c; k < CLS_TC * 64; k += di) s_dbc[k] = 0.f;

    // this channel's constants
    float cw[CLS_MAX_CONV], A[CLS_MAX_STATE], wdt[CLS_MAX_RANK], h[CLS_MAX_STATE], xh[CLS_MAX_CONV];
#pragma unroll
    for (int j = 0; j < CLS_MAX_CONV; ++j) {
        const int src = j - (CLS_MAX_CONV - v.d_conv); // taps right-aligned: the last one meets the current token
        cw[j] = src >= 0 ? v.conv_w[c * v.d_conv + src] : 0.f;
        xh[j] = 0.f;
    }
#pragma unroll
    for (int n = 0; n < CLS_MAX_STATE; ++n) {
        A[n] = n < v.d_state ? -expf(v.a_log[c * v.d_state + n]) * 1.44269504088896f : 0.f; // times log2(e): decay = 2^(Delta A)
        h[n] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < CLS_MAX_RANK; ++r) wdt[r] = r < v.dt_rank ? v.w_dt[r * di + c] : 0.f;
    const float cb = v.conv_b[c], bdt = v.b_dt[c], D = v.d[c];
    float pooled = 0.f;

    // The input projection's two values of this channel for one chunk of tokens, gathered from the
    // table.  Two loads depend on each other (token id, then table row), so both run ahead: lane t of
    // every wave holds the id of token t of the chunk after next while the next chunk's rows fly.
    float nx[CLS_TC], nz[CLS_TC];
    bool bad = false;
    int idv = 0;
    auto load_ids = [&](int t0) {
        const int t = t0 + (lane & (CLS_TC - 1));
        idv = t < L ? tok[t] : 0;
    };
    auto gather = [&](int t0) {
#pragma unroll
        for (int t = 0; t < CLS_TC; ++t) {
            nx[t] = nz[t] = 0.f;
            const int id = __builtin_amdgcn_readlane(idv, t);
            if (t0 + t < L) {
                if ((unsigned)id < (unsigned)v.vocab) {
                    const float *row = v.table + (size_t)id * 2 * di + c;
                    nx[t] = row[0];
                    nz[t] = row[di];
                } else
                    bad = true;
            }
        }
    };
    load_ids(0);
    gather(0);
    load_ids(CLS_TC);

    for (int t0 = 0; t0 < L; t0 += CLS_TC) {
        const int nt = min(CLS_TC, L - t0);
        float x[CLS_TC], z[CLS_TC];
        // causal depthwise convolution and SiLU: no dependence on the state, so the whole chunk at once
#pragma unroll
        for (int t = 0; t < CLS_TC; ++t) {
            xh[0] = xh[1]; xh[1] = xh[2]; xh[2] = xh[3]; xh[3] = nx[t];
            float pre = cb;
#pragma unroll
            for (int j = 0; j < CLS_MAX_CONV; ++j) pre = fmaf(cw[j], xh[j], pre);
            x[t] = pre * __builtin_amdgcn_rcpf(1.f + __expf(-pre));
            z[t] = nz[t];
        }
        *(float4 *)(s_x + c * CLS_TC) = make_float4(x[0], x[1], x[2], x[3]);
        *(float4 *)(s_x + c * CLS_TC + 4) = make_float4(x[4], x[5], x[6], x[7]);
        gather(t0 + CLS_TC); // the next chunk's rows fly while this one is worked on
        load_ids(t0 + 2 * CLS_TC);
        __syncthreads();

        // (r, B, C) = x W_x for the chunk: each wave sums its 64 channels for output `lane`
        if (lane < J) {
            float p[CLS_TC];
#pragma unroll
            for (int t = 0; t < CLS_TC; ++t) p[t] = 0.f;
            const float *wx = s_wx + (size_t)wave * 64 * J + lane;
            const float *xs = s_x + (size_t)wave * 64 * CLS_TC;
#pragma unroll 4
            for (int k = 0; k < 64; ++k) {
                const float w = wx[k * J];
                const float4 a = *(const float4 *)(xs + k * CLS_TC), b = *(const float4 *)(xs + k * CLS_TC + 4);
                p[0] = fmaf(a.x, w, p[0]); p[1] = fmaf(a.y, w, p[1]); p[2] = fmaf(a.z, w, p[2]); p[3] = fmaf(a.w, w, p[3]);
                p[4] = fmaf(b.x, w, p[4]); p[5] = fmaf(b.y, w, p[5]); p[6] = fmaf(b.z, w, p[6]); p[7] = fmaf(b.w, w, p[7]);
            }
#pragma unroll
            for (int t = 0; t < CLS_TC; ++t) s_part[(wave * CLS_TC + t) * 64 + lane] = p[t];
        }
        __syncthreads();
        for (int q = c; q < CLS_TC * 64; q += di) {
            const int j = q & 63;
            if (j < J) {
                float p = 0.f;
                for (int w = 0; w < waves; ++w) p += s_part[w * CLS_TC * 64 + q];
                const int slot = j < v.dt_rank ? j : (j < v.dt_rank + v.d_state ? 16 + j - v.dt_rank : 32 + j - v.dt_rank - v.d_state);
                s_dbc[(q & ~63) + slot] = p;
            }
        }
        __syncthreads();

        // the state update, token by token, all in this thread's registers
#pragma unroll
        for (int t = 0; t < CLS_TC; ++t) {
            if (t >= nt) break; // uniform over the block
            const float *dbc = s_dbc + t * 64;
            float dt = bdt;
#pragma unroll
            for (int r = 0; r < CLS_MAX_RANK; ++r) dt = fmaf(dbc[r], wdt[r], dt);
            // softplus = log1p(e^dt): log(u) e / (u - 1) with u = 1 + e undoes the rounding of u (steps are ~1e-3..0.1)
            const float e = __expf(dt), u = 1.f + e;
            const float delta = dt > 20.f ? dt : (u == 1.f ? e : logf(u) * e * __builtin_amdgcn_rcpf(u - 1.f));
            const float dx = delta * x[t];
            float acc = 0.f;
#pragma unroll
            for (int n = 0; n < CLS_MAX_STATE; ++n) {
                h[n] = fmaf(__builtin_amdgcn_exp2f(delta * A[n]), h[n], dx * dbc[16 + n]);
                acc = fmaf(dbc[32 + n], h[n], acc);
            }
            pooled += (acc + D * x[t]) * z[t] * __builtin_amdgcn_rcpf(1.f + __expf(-z[t]));
        }
    }
    if (bad) s_bad = 1;

    // mean over tokens, output projection, linear layer, arg max
    __syncthreads();
    s_x[c] = L > 0 ? pooled / (float)L : 0.f;
    __syncthreads();
    for (int m = c; m < dm; m += di) {
        float o = 0.f;
        for (int k = 0; k < di; ++k) o = fmaf(s_x[k], v.w_out[(size_t)k * dm + m], o);
        s_o[m] = o;
    }
    __syncthreads();
    float *s_logit = s_o + dm;
    for (int k = c; k < v.n_classes; k += di) {
        float o = v.b_fc[k];
        for (int m = 0; m < dm; ++m) o = fmaf(s_o[m], v.w_fc[(size_t)k * dm + m], o);
        s_logit[k] = o;
        if (logits) logits[(size_t)i * v.n_classes + k] = o;
    }
    __syncthreads();
    if (c == 0) {
        int best = 0;
        for (int k = 1; k < v.n_classes; ++k)
            if (s_logit[k] > s_logit[best]) best = k;
        draft_id[i] = s_bad ? -1 : best;
    }
}

// ---------------------------------------------------------------- C ABI

extern "C" int sd_classifier_create(const sd_classifier_shape *s, const sd_classifier_weights *w, sd_classifier **out)
{
    if (!s || !w || !out) return sd_fail(SD_EINVAL, "sd_classifier_create: null argument");
    *out = nullptr;
    if (s->vocab < 1 || s->n_classes < 1 || s->n_classes > CLS_MAX_CLASSES)
        return sd_fail(SD_EINVAL, "sd_classifier_create: vocab >= 1 and 1 <= n_classes <= 64 required");
    if (s->d_model < 1 || s->d_model > CLS_MAX_MODEL || s->d_inner < 64 || s->d_inner > CLS_MAX_INNER || s->d_inner % 64)
        return sd_fail(SD_EINVAL, "sd_classifier_create: d_model in [1, 512] and d_inner a multiple of 64 in [64, 512] required");
    if (s->d_state < 1 || s->d_state > CLS_MAX_STATE || s->dt_rank < 1 || s->dt_rank > CLS_MAX_RANK || s->d_conv < 1 ||
        s->d_conv > CLS_MAX_CONV)
        return sd_fail(SD_EINVAL, "sd_classifier_create: d_state, dt_rank in [1, 16] and d_conv in [1, 4] required");
    const float *src[12] = {w->emb, w->w_in, w->conv_w, w->conv_b, w->w_x, w->w_dt, w->b_dt, w->a_log, w->d, w->w_out,
                            w->w_fc, w->b_fc};
    for (const float *p : src)
        if (!p) return sd_fail(SD_EINVAL, "sd_classifier_create: null weight pointer");
    const size_t J = (size_t)s->dt_rank + 2 * (size_t)s->d_state;
    const size_t lds_bytes = cls_lds_floats(s->d_inner, (int)J, s->d_model) * sizeof(float);
    if (lds_bytes > CLS_LDS_LIMIT)
        return sd_fail(SD_EINVAL, "sd_classifier_create: d_inner * (dt_rank + 2 d_state) does not fit the 64 KB of LDS "
                                  "the per-token projection is staged in");
    // slot 0 holds the table emb W_in; slot 1 is unused once the table is built (emb and W_in go to a
    // temporary allocation), the rest are copies of the caller's arrays.
    const size_t cols = 2 * (size_t)s->d_inner;
    const size_t count[12] = {(size_t)s->vocab * cols, 0,
                              (size_t)s->d_inner * s->d_conv, (size_t)s->d_inner, (size_t)s->d_inner * J,
                              (size_t)s->dt_rank * s->d_inner, (size_t)s->d_inner, (size_t)s->d_inner * s->d_state,
                              (size_t)s->d_inner, (size_t)s->d_inner * s->d_model, (size_t)s->n_classes * s->d_model,
                              (size_t)s->n_classes};
    size_t total = 0, off[12];
    for (int k = 0; k < 12; ++k) { off[k] = total; total += (count[k] * sizeof(float) + 255) & ~(size_t)255; }
    const size_t emb_bytes = (size_t)s->vocab * s->d_model * sizeof(float), emb_slot = (emb_bytes + 255) & ~(size_t)255;
    const size_t win_bytes = (size_t)s->d_model * cols * sizeof(float);

    sd_classifier *c = new sd_classifier();
    c->v.vocab = s->vocab; c->v.d_model = s->d_model; c->v.d_inner = s->d_inner; c->v.d_state = s->d_state;
    c->v.dt_rank = s->dt_rank; c->v.d_conv = s->d_conv; c->v.n_classes = s->n_classes;
    c->lds_bytes = lds_bytes;
    c->mem = nullptr;
    void *tmp = nullptr;
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = hipMalloc(&c->mem, total);
    if (e == hipSuccess) e = hipMalloc(&tmp, emb_slot + win_bytes);
    const float **dst[12] = {&c->v.table, nullptr, &c->v.conv_w, &c->v.conv_b, &c->v.w_x, &c->v.w_dt, &c->v.b_dt,
                             &c->v.a_log, &c->v.d, &c->v.w_out, &c->v.w_fc, &c->v.b_fc};
    for (int k = 0; k < 12 && e == hipSuccess; ++k) {
        if (!dst[k]) continue;
        *dst[k] = (const float *)((char *)c->mem + off[k]);
        if (k >= 2) e = hipMemcpy((char *)c->mem + off[k], src[k], count[k] * sizeof(float), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipMemcpy(tmp, w->emb, emb_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy((char *)tmp + emb_slot, w->w_in, win_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(classifier_table_kernel, dim3(s->vocab), dim3(256), 0, (hipStream_t)0, (const float *)tmp,
                           (const float *)((char *)tmp + emb_slot), s->d_model, (int)cols, (float *)c->mem);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (tmp) (void)hipFree(tmp);
    if (e != hipSuccess) {
        if (c->mem) (void)hipFree(c->mem);
        delete c;
        return sd_fail(SD_EHIP, std::string("sd_classifier_create: ") + hipGetErrorString(e));
    }
    *out = c;
    return SD_OK;
}

extern "C" void sd_classifier_destroy(sd_classifier *c)
{
    if (!c) return;
    (void)hipFree(c->mem);
    delete c;
}

extern "C" int sd_route_classifier(const sd_classifier *c, const int32_t *tokens, const int32_t *lens, int32_t n,
                                   int32_t max_len, float *logits, int32_t *draft_id, void *stream)
{
    if (!c || !tokens || !lens || !draft_id) return sd_fail(SD_EINVAL, "sd_route_classifier: null argument");
    if (n < 1 || max_len < 1) return sd_fail(SD_EINVAL, "sd_route_classifier: non-positive size");
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != c->device)
        return sd_fail(SD_EINVAL, "sd_route_classifier: the classifier was created on another device");
    hipLaunchKernelGGL(classifier_kernel, dim3(n), dim3(c->v.d_inner), c->lds_bytes, (hipStream_t)stream, c->v, tokens,
                       lens, max_len, logits, draft_id);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sd_fail(SD_EHIP, std::string("sd_route_classifier: ") + hipGetErrorString(e));
    return SD_OK;
}
