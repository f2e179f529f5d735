// C ABI of libsd and the host-side launch schedule of one decoder forward.
// See include/sd.h for the contract of every entry point.
#include <math.h>
#include <string.h>

#include <algorithm>

#include "sd_internal.h"
#include <cmath>

static thread_local std::string g_err;
int g_force_generic = 0;
static int g_norm_fold = 0; // option "norm_fold"

void sd_set_error(const std::string &s) { g_err = s; }
int sd_fail(int code, const std::string &s)
{
    g_err = s;
    return code;
}

extern "C" const char *sd_last_error(void) { return g_err.c_str(); }

// ---------------------------------------------------------------- per-kernel timing (option "profile")
// When enabled, every launch of the forward is bracketed by two HIP events on the
// stream it runs on; sd_profile_read folds them into per-kernel-class totals.
enum ProfTag { T_PLAN, T_EMBED, T_RMSNORM, T_QKV, T_ROPE, T_ATTN, T_OPROJ, T_GATEUP, T_DOWN, T_LMHEAD, T_SAMPLE, T_TAIL, T_LORA, T_COUNT };
static const char *g_tag_names[T_COUNT] = {"plan", "embed", "rmsnorm", "gemm_qkv", "rope_append", "attention", "gemm_o",
                                           "gemm_gateup", "gemm_down", "gemm_lmhead", "draft_sample", "verify_tail", "lora"};
struct ProfRec {
    int tag;
    hipEvent_t e0, e1;
};
static int g_profile = 0;
static std::vector<ProfRec> g_recs;
static std::vector<hipEvent_t> g_pool;
static int g_prof_count[T_COUNT];
static float g_prof_ms[T_COUNT];

static hipEvent_t prof_event()
{
    hipEvent_t e;
    if (!g_pool.empty()) {
        e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct ProfScope {
    hipStream_t s;
    int tag;
    hipEvent_t e0, e1;
    ProfScope(int tag_, hipStream_t s_) : s(s_), tag(tag_), e0(nullptr), e1(nullptr)
    {
        if (!g_profile) return;
        e0 = prof_event();
        e1 = prof_event();
        if (e0) (void)hipEventRecord(e0, s);
    }
    ~ProfScope()
    {
        if (!e0 || !e1) return;
        (void)hipEventRecord(e1, s);
        g_recs.push_back({tag, e0, e1});
    }
};

static void prof_fold()
{
    for (auto &r : g_recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.e1) == hipSuccess && hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
            g_prof_count[r.tag]++;
            g_prof_ms[r.tag] += ms;
        }
        g_pool.push_back(r.e0);
        g_pool.push_back(r.e1);
    }
    g_recs.clear();
}

extern "C" int sd_profile_read(int32_t idx, const char **name, int32_t *count, float *total_ms)
{
    if (idx < 0 || idx >= T_COUNT || !name || !count || !total_ms) return sd_fail(SD_EINVAL, "sd_profile_read: bad index");
    prof_fold();
    *name = g_tag_names[idx];
    *count = g_prof_count[idx];
    *total_ms = g_prof_ms[idx];
    return SD_OK;
}

extern "C" int sd_set_option(const char *name, int32_t value)
{
    if (!name) return sd_fail(SD_EINVAL, "sd_set_option: null name");
    if (!strcmp(name, "force_generic")) { // bit 0: GEMMs, bit 1: attention, bit 2: draft sampler that reads whole rows,
                                          // bit 3: output projection as a launch of its own; 1 means all
        g_force_generic = value == 1 ? 15 : value;
        return SD_OK;
    }
    if (!strcmp(name, "gemm_splits")) { // value = mode*100 + K splits of the few-row / row-blocked GEMM (0 = automatic)
        const int mode = value / 100, ks = value % 100;
        if (value < 0 || mode > 2 || ks > 8) return sd_fail(SD_EINVAL, "sd_set_option: bad gemm_splits value");
        g_force_splits[mode] = ks;
        return SD_OK;
    }
    if (!strcmp(name, "gemm_tile_cols")) { // weight rows per block of the row-blocked GEMM: 128, 192, 256, or 0 = automatic
        if (value != 0 && value != 128 && value != 192 && value != 256)
            return sd_fail(SD_EINVAL, "sd_set_option: gemm_tile_cols is 0, 128, 192 or 256");
        g_force_tile_cols = value;
        return SD_OK;
    }
    if (!strcmp(name, "norm_fold")) { // add + RMSNorm split between producer and consumer GEMM: 0 or 1 = wherever the shapes
                                      // allow (the default), 2 = never
        if (value < 0 || value > 2) return sd_fail(SD_EINVAL, "sd_set_option: norm_fold is 0, 1 or 2");
        g_norm_fold = value;
        return SD_OK;
    }
    if (!strcmp(name, "rope_group")) { // RoPE + cache append of the split attention path: 1 = one block per (head, row group)
                                       // with 16-byte stores (default), 0 = one block per row
        if (value != 0 && value != 1) return sd_fail(SD_EINVAL, "sd_set_option: rope_group is 0 or 1");
        g_rope_group = value;
        return SD_OK;
    }
    if (!strcmp(name, "prefill_attn")) { // attention of prefill forwards: 1 = row groups of a prompt share staged K / V tiles
                                         // (default), 0 = the split kernel, one set of blocks per group
        if (value != 0 && value != 1) return sd_fail(SD_EINVAL, "sd_set_option: prefill_attn is 0 or 1");
        g_prefill_attn = value;
        return SD_OK;
    }
    if (!strcmp(name, "attn_waves")) { // waves per block of the fused attention kernel: 4, 8, or 0 = automatic
        if (value != 0 && value != 4 && value != 8) return sd_fail(SD_EINVAL, "sd_set_option: attn_waves is 0, 4 or 8");
        g_force_attn_waves = value;
        return SD_OK;
    }
    if (!strcmp(name, "stream_read_nt")) { // pattern of sd_debug_stream_read: 1 = contiguous ranges, nontemporal hint (default);
                                           // 0 = grid-strided; + 2 = checking mode (XOR of every word read is folded into the scratch word)
        if (value < 0 || value > 3) return sd_fail(SD_EINVAL, "sd_set_option: stream_read_nt is 0..3");
        g_stream_read_nt = value;
        return SD_OK;
    }
    if (!strcmp(name, "profile")) { // 1: start a fresh measurement, 0: stop recording (totals stay readable)
        prof_fold();
        if (value) {
            for (int i = 0; i < T_COUNT; i++) g_prof_count[i] = 0, g_prof_ms[i] = 0.f;
        }
        g_profile = value;
        return SD_OK;
    }
    return sd_fail(SD_EINVAL, std::string("sd_set_option: unknown option ") + name);
}

// ---------------------------------------------------------------- candidate-count policy (Equation 1)
extern "C" double sd_eq1_speedup(double alpha, int32_t gamma, double c)
{
    if (!(alpha >= 0.0 && alpha <= 1.0) || !(c >= 0.0) || gamma < 0) return std::nan("");
    // tokens per step: 1 + alpha + ... + alpha^gamma, summed directly (no cancellation near alpha = 1)
    double tokens = 0.0, term = 1.0;
    for (int i = 0; i <= gamma; i++) {
        tokens += term;
        term *= alpha;
    }
    return tokens / (gamma * c + 1.0);
}

extern "C" int32_t sd_choose_gamma(double alpha, double c, int32_t gamma_max, double *speedup)
{
    if (!(alpha >= 0.0 && alpha <= 1.0) || !(c >= 0.0) || gamma_max < 0 || gamma_max > SD_MAX_GAMMA) {
        sd_fail(SD_EINVAL, "sd_choose_gamma: alpha in [0,1], c >= 0, 0 <= gamma_max <= 15");
        return -1;
    }
    int best = 0;
    double best_v = sd_eq1_speedup(alpha, 0, c);
    for (int g = 1; g <= gamma_max; g++) {
        const double v = sd_eq1_speedup(alpha, g, c);
        if (v > best_v) best = g, best_v = v;
    }
    if (speedup) *speedup = best_v;
    return best;
}

extern "C" double sd_alpha_hat(const int32_t *n_accepted, int32_t n_steps, int32_t gamma)
{
    if (!n_accepted || n_steps < 1 || gamma < 1) return std::nan("");
    long accepted = 0, examined = 0;
    for (int i = 0; i < n_steps; i++) {
        const int a = n_accepted[i];
        if (a < 0 || a > gamma) return std::nan("");
        accepted += a;
        examined += a < gamma ? a + 1 : gamma;
    }
    return examined ? (double)accepted / (double)examined : std::nan("");
}

// ---------------------------------------------------------------- model
static size_t attn_part_floats(const sd_model_config &c) { return (size_t)3072 * 16 * (c.head_dim + 2); }

extern "C" int sd_load_model(const sd_model_config *cfg, const sd_weights *w, sd_model **out)
{
    if (!cfg || !w || !out) return sd_fail(SD_EINVAL, "sd_load_model: null argument");
    const sd_model_config &c = *cfg;
    if (c.n_layers < 1 || c.d_model < 1 || c.n_heads < 1 || c.d_ffn < 1 || c.vocab < 1)
        return sd_fail(SD_EINVAL, "sd_load_model: non-positive dimension");
    if (c.n_heads * c.head_dim != c.d_model) return sd_fail(SD_EINVAL, "sd_load_model: n_heads*head_dim != d_model");
    if (c.head_dim != 16 && c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128)
        return sd_fail(SD_EINVAL, "sd_load_model: head_dim must be 16, 32, 64 or 128");
    if (c.vocab % 4 != 0) return sd_fail(SD_EINVAL, "sd_load_model: vocab must be a multiple of 4");
    if (c.vocab > 262144) // the samplers search 64 segments of 4096 entries
        return sd_fail(SD_EINVAL, "sd_load_model: vocab above 262144");
    if (c.dtype != SD_FP32 && c.dtype != SD_BF16) return sd_fail(SD_EINVAL, "sd_load_model: bad dtype");
    if (c.max_rows < 2 || c.max_pos < 2) return sd_fail(SD_EINVAL, "sd_load_model: max_rows/max_pos too small");
    if (!(c.rope_base > 1.f) || !(c.rms_eps >= 0.f)) return sd_fail(SD_EINVAL, "sd_load_model: bad rope_base/rms_eps");
    if (!w->embed || !w->lm_head || !w->final_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->wgate ||
        !w->wup || !w->wdown || !w->norm_attn || !w->norm_ffn)
        return sd_fail(SD_EINVAL, "sd_load_model: null weight pointer");
    for (int l = 0; l < c.n_layers; l++)
        if (!w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->wgate[l] || !w->wup[l] || !w->wdown[l] ||
            !w->norm_attn[l] || !w->norm_ffn[l])
            return sd_fail(SD_EINVAL, "sd_load_model: null per-layer weight pointer");
    sd_model *m = new sd_model();
    m->cfg = c;
    m->esz = c.dtype == SD_BF16 ? 2 : 4;
    m->lora_n = 0;
    m->lora_rank = 0;
    m->lora_scale = 0.f;
    m->lora_mem = nullptr;
    // ---- weights: one arena owned by the model.  bf16 matrices whose shape allows it are re-ordered into
    // 16 x 128 tiles on the way (the streaming GEMMs read those); everything else is copied as is.
    {
        const size_t d = c.d_model, F = c.d_ffn, V = c.vocab, esz = m->esz;
        auto can_tile = [&](size_t N, size_t K) { return c.dtype == SD_BF16 && N % 16 == 0 && K % 128 == 0; };
        m->tiled_dd = can_tile(d, d);
        m->tiled_fd = can_tile(F, d);
        m->tiled_df = can_tile(d, F);
        m->tiled_lm = can_tile(V, d);
        auto pad = [](size_t b) { return (b + 255) & ~(size_t)255; };
        const size_t b_dd = pad(d * d * esz), b_fd = pad(F * d * esz), b_vd = pad(V * d * esz), b_g = pad(d * 4);
        const size_t total = 2 * b_vd + b_g + (size_t)c.n_layers * (4 * b_dd + 3 * b_fd + 2 * b_g);
        // weights that cannot stay in the 256 MB memory-side cache from one forward to the next are streamed past it
        m->stream_nt = total > ((size_t)256 << 20);
        hipError_t we = hipMalloc(&m->wmem, total);
        if (we != hipSuccess) {
            delete m;
            return sd_fail(SD_EHIP, std::string("sd_load_model: hipMalloc(weights): ") + hipGetErrorString(we));
        }
        char *cur = (char *)m->wmem;
        auto put = [&](const void *src, size_t N, size_t K, size_t bytes, int tiled) -> const void * {
            void *dst = cur;
            cur += bytes;
            if (we != hipSuccess) return dst;
            if (tiled) we = launch_retile_bf16(0, src, dst, (int)N, (int)K);
            else we = hipMemcpyAsync(dst, src, N * K * esz, hipMemcpyDeviceToDevice, 0);
            return dst;
        };
        auto put_gain = [&](const float *src) -> const float * {
            void *dst = cur;
            cur += b_g;
            if (we == hipSuccess) we = hipMemcpyAsync(dst, src, d * 4, hipMemcpyDeviceToDevice, 0);
            return (const float *)dst;
        };
        m->embed = put(w->embed, V, d, b_vd, 0); // gathered by row: stays row-major
        m->lm_head = put(w->lm_head, V, d, b_vd, m->tiled_lm);
        m->final_norm = put_gain(w->final_norm);
        for (int l = 0; l < c.n_layers; l++) {
            m->wq.push_back(put(w->wq[l], d, d, b_dd, m->tiled_dd));
            m->wk.push_back(put(w->wk[l], d, d, b_dd, m->tiled_dd));
            m->wv.push_back(put(w->wv[l], d, d, b_dd, m->tiled_dd));
            m->wo.push_back(put(w->wo[l], d, d, b_dd, m->tiled_dd));
            m->wgate.push_back(put(w->wgate[l], F, d, b_fd, m->tiled_fd));
            m->wup.push_back(put(w->wup[l], F, d, b_fd, m->tiled_fd));
            m->wdown.push_back(put(w->wdown[l], d, F, b_fd, m->tiled_df));
            m->norm_attn.push_back(put_gain(w->norm_attn[l]));
            m->norm_ffn.push_back(put_gain(w->norm_ffn[l]));
        }
        if (we == hipSuccess) we = hipStreamSynchronize(0);
        if (we != hipSuccess) {
            (void)hipFree(m->wmem);
            delete m;
            return sd_fail(SD_EHIP, std::string("sd_load_model: weight copy: ") + hipGetErrorString(we));
        }
    }
    m->last_lm_rows = 0;
    size_t M = c.max_rows, d = c.d_model;
    m->part_floats = attn_part_floats(c);
    hipError_t e = hipSuccess;
    auto alloc = [&](void **p, size_t bytes) {
        if (e == hipSuccess) e = hipMalloc(p, bytes);
    };
    m->x = nullptr;
    const size_t planes = c.dtype == SD_BF16 ? 2 : 1; // bf16 activations are stored as hi + lo
    m->plane_d = M * d;
    m->plane_f = M * (size_t)c.d_ffn;
    alloc((void **)&m->x, M * d * 4);
    const size_t act_pad = (size_t)SD_ACT_PAD_ROWS * 128 * m->esz; // slack read (never used) by the row-blocked GEMM
    // (the per-block sums of squares of a split norm sit behind the operand rows their consumer reads anyway: the
    // same pages)
    const size_t abuf_bytes = (planes * M * d * m->esz + act_pad + 255) & ~(size_t)255;
    alloc(&m->abuf, abuf_bytes + (size_t)SD_NORMFOLD_MAX_BLOCKS * 32 * sizeof(float));
    alloc((void **)&m->qkv, M * 3 * d * 4);
    alloc(&m->qbuf, planes * M * d * m->esz + act_pad);
    alloc(&m->obuf, planes * M * d * m->esz + act_pad);
    alloc(&m->act, planes * M * (size_t)c.d_ffn * m->esz + act_pad);
    alloc((void **)&m->logits, M * (size_t)c.vocab * 4);
    alloc((void **)&m->vstats, M * 3 * sizeof(float));
    alloc((void **)&m->lm_stats, M * (size_t)(c.vocab / 32 + 1) * 3 * sizeof(float));
    m->ss_part = e == hipSuccess ? (float *)((char *)m->abuf + abuf_bytes) : nullptr;
    m->lm_stats_nb = 0;
    alloc((void **)&m->part, m->part_floats * 4);
    m->gpart_q_floats = 8 * M * 3 * d;
    // (a small model's attention blocks may leave one slab per head instead: see launch_attn_fused_bf16)
    m->gpart_r_floats = (size_t)(d <= 1024 && c.n_heads <= SD_OPROJ_MAX_HEADS ? std::max(8, c.n_heads) : 8) * M * d;
    alloc((void **)&m->gpart_q, m->gpart_q_floats * 4);
    alloc((void **)&m->gpart_r, m->gpart_r_floats * 4);
    alloc((void **)&m->rope, (size_t)c.max_pos * (c.head_dim / 2) * sizeof(float2));
    alloc((void **)&m->plan_mem, (5 * M + 4 * M) * sizeof(int32_t));
    if (e != hipSuccess) {
        sd_free_model(m);
        return sd_fail(SD_EHIP, std::string("sd_load_model: hipMalloc: ") + hipGetErrorString(e));
    }
    int32_t *pm = m->plan_mem;
    m->plan.row_tok = pm;
    m->plan.row_pos = pm + M;
    m->plan.row_b = pm + 2 * M;
    m->plan.row_valid = pm + 3 * M;
    m->plan.lm_row = pm + 4 * M;
    m->plan.seq_b = pm + 5 * M;
    m->plan.seq_kv0 = pm + 6 * M;
    m->plan.seq_nq = pm + 7 * M;
    m->plan.seq_order = pm + 8 * M;
    // rotary table in double on the host: angle = pos * base^(-2i/hd)
    int half = c.head_dim / 2;
    std::vector<float2> tab((size_t)c.max_pos * half);
    for (int i = 0; i < half; i++) {
        double theta = pow((double)c.rope_base, -2.0 * i / c.head_dim);
        for (int p = 0; p < c.max_pos; p++) {
            double a = p * theta;
            tab[(size_t)p * half + i] = make_float2((float)cos(a), (float)sin(a));
        }
    }
    SD_HIP(hipMemcpy(m->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
    SD_HIP(hipDeviceSynchronize());
    *out = m;
    return SD_OK;
}

extern "C" int sd_free_model(sd_model *m)
{
    if (!m) return SD_OK;
    (void)hipDeviceSynchronize();
    (void)hipFree(m->x);
    (void)hipFree(m->abuf);
    (void)hipFree(m->qkv);
    (void)hipFree(m->qbuf);
    (void)hipFree(m->obuf);
    (void)hipFree(m->act);
    (void)hipFree(m->logits);
    (void)hipFree(m->vstats);
    (void)hipFree(m->lm_stats);
    (void)hipFree(m->part);
    (void)hipFree(m->gpart_q);
    (void)hipFree(m->gpart_r);
    (void)hipFree(m->rope);
    (void)hipFree(m->plan_mem);
    (void)hipFree(m->wmem);
    (void)hipFree(m->lora_mem);
    delete m;
    return SD_OK;
}

// ---------------------------------------------------------------- low-rank adapters (Section 2.3)
extern "C" int sd_model_set_lora(sd_model *m, const sd_lora_weights *w)
{
    if (!m || !w) return sd_fail(SD_EINVAL, "sd_model_set_lora: null argument");
    if (w->n_adapters < 0 || (w->n_adapters > 0 && (w->rank < 1 || w->rank > 16)))
        return sd_fail(SD_EINVAL, "sd_model_set_lora: n_adapters >= 0, 1 <= rank <= 16");
    if (m->cfg.d_model > 8192) return sd_fail(SD_EINVAL, "sd_model_set_lora: d_model above 8192");
    SD_HIP(hipDeviceSynchronize());
    (void)hipFree(m->lora_mem);
    m->lora_mem = nullptr;
    m->lora_n = 0;
    for (int p = 0; p < 4; p++) m->lora_a[p].clear(), m->lora_b[p].clear();
    if (w->n_adapters == 0) return SD_OK;
    const int L = m->cfg.n_layers, n = w->n_adapters, r = w->rank;
    const size_t d = m->cfg.d_model, per = (size_t)n * r * d; // floats of one factor of one layer
    const void *const *src_a[4] = {w->a_q, w->a_k, w->a_v, w->a_o}, *const *src_b[4] = {w->b_q, w->b_k, w->b_v, w->b_o};
    size_t total = 0;
    for (int p = 0; p < 4; p++) {
        if ((src_a[p] == nullptr) != (src_b[p] == nullptr))
            return sd_fail(SD_EINVAL, "sd_model_set_lora: a projection needs both factors or neither");
        if (src_a[p]) total += 2 * per * L;
    }
    if (!total) return SD_OK;
    SD_HIP(hipMalloc(&m->lora_mem, total * sizeof(float)));
    std::vector<float> host(per);
    float *dst = (float *)m->lora_mem;
    auto upload = [&](const void *src) -> hipError_t { // one factor of one layer: to fp32, then to the device
        if (m->cfg.dtype == SD_BF16) {
            const uint16_t *b = (const uint16_t *)src;
            for (size_t i = 0; i < per; i++) {
                const uint32_t u = (uint32_t)b[i] << 16;
                memcpy(&host[i], &u, 4);
            }
        } else {
            memcpy(host.data(), src, per * sizeof(float));
        }
        return hipMemcpy(dst, host.data(), per * sizeof(float), hipMemcpyHostToDevice);
    };
    for (int p = 0; p < 4; p++) {
        m->lora_a[p].assign(L, nullptr);
        m->lora_b[p].assign(L, nullptr);
        if (!src_a[p]) continue;
        for (int l = 0; l < L; l++) {
            if (!src_a[p][l] || !src_b[p][l]) return sd_fail(SD_EINVAL, "sd_model_set_lora: null factor of a layer");
            SD_HIP(upload(src_a[p][l]));
            m->lora_a[p][l] = dst;
            dst += per;
            SD_HIP(upload(src_b[p][l]));
            m->lora_b[p][l] = dst;
            dst += per;
        }
    }
    m->lora_n = n;
    m->lora_rank = r;
    m->lora_scale = w->scale;
    return SD_OK;
}

// ---------------------------------------------------------------- context
extern "C" int sd_ctx_create(int32_t batch, const int32_t *caps, sd_ctx **out)
{
    if (batch < 1 || !caps || !out) return sd_fail(SD_EINVAL, "sd_ctx_create: bad argument");
    sd_ctx *c = new sd_ctx();
    c->B = batch;
    c->n_slots = 0;
    c->len_upper = 0;
    int64_t tot = 0;
    for (int b = 0; b < batch; b++) {
        if (caps[b] < 1) {
            delete c;
            return sd_fail(SD_EINVAL, "sd_ctx_create: capacity < 1");
        }
        int32_t cp = (caps[b] + 63) / 64 * 64; // 64-token granules keep cache rows 128-byte aligned
        c->cap.push_back(cp);
        c->off.push_back(tot);
        tot += cp;
    }
    c->total_cap = tot;
    c->max_cap = *std::max_element(c->cap.begin(), c->cap.end());
    for (int s = 0; s < SD_MAX_SLOTS; s++) c->models[s] = nullptr, c->kcache[s] = c->vcache[s] = nullptr;
    hipError_t e = hipMalloc((void **)&c->d_off, sizeof(int64_t) * batch);
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_cap, sizeof(int32_t) * batch);
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_tokens, sizeof(int32_t) * tot);
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_ntok, sizeof(int32_t) * batch);
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_kvlen, sizeof(int32_t) * batch * SD_MAX_SLOTS);
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_status, sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_adapter, sizeof(int32_t) * batch * SD_MAX_SLOTS);
    c->use_gamma = 0;
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_gamma, sizeof(int32_t) * batch);
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_policy, sizeof(int32_t) * batch * 2);
    if (e != hipSuccess) {
        delete c;
        return sd_fail(SD_EHIP, std::string("sd_ctx_create: hipMalloc: ") + hipGetErrorString(e));
    }
    SD_HIP(hipMemcpy(c->d_off, c->off.data(), sizeof(int64_t) * batch, hipMemcpyHostToDevice));
    SD_HIP(hipMemcpy(c->d_cap, c->cap.data(), sizeof(int32_t) * batch, hipMemcpyHostToDevice));
    SD_HIP(hipMemset(c->d_tokens, 0, sizeof(int32_t) * tot));
    SD_HIP(hipMemset(c->d_ntok, 0, sizeof(int32_t) * batch));
    SD_HIP(hipMemset(c->d_kvlen, 0, sizeof(int32_t) * batch * SD_MAX_SLOTS));
    SD_HIP(hipMemset(c->d_status, 0, sizeof(int32_t)));
    SD_HIP(hipMemset(c->d_adapter, 0xff, sizeof(int32_t) * batch * SD_MAX_SLOTS)); // -1: no adapter
    SD_HIP(hipMemset(c->d_gamma, 0, sizeof(int32_t) * batch));
    SD_HIP(hipMemset(c->d_policy, 0, sizeof(int32_t) * batch * 2));
    SD_HIP(hipDeviceSynchronize());
    *out = c;
    return SD_OK;
}

extern "C" int sd_ctx_free(sd_ctx *c)
{
    if (!c) return SD_OK;
    (void)hipDeviceSynchronize();
    for (int s = 0; s < c->n_slots; s++) {
        (void)hipFree(c->kcache[s]);
        (void)hipFree(c->vcache[s]);
    }
    (void)hipFree(c->d_off);
    (void)hipFree(c->d_cap);
    (void)hipFree(c->d_tokens);
    (void)hipFree(c->d_ntok);
    (void)hipFree(c->d_kvlen);
    (void)hipFree(c->d_status);
    (void)hipFree(c->d_adapter);
    (void)hipFree(c->d_gamma);
    (void)hipFree(c->d_policy);
    delete c;
    return SD_OK;
}

static int find_slot(const sd_ctx *c, const sd_model *m)
{
    for (int s = 0; s < c->n_slots; s++)
        if (c->models[s] == m) return s;
    return -1;
}

extern "C" int sd_ctx_set_adapters(sd_ctx *c, sd_model *m, const int32_t *adapter_ids)
{
    if (!c || !m || !adapter_ids) return sd_fail(SD_EINVAL, "sd_ctx_set_adapters: null argument");
    const int slot = find_slot(c, m);
    if (slot < 0) return sd_fail(SD_EINVAL, "sd_ctx_set_adapters: model not attached to this context");
    for (int b = 0; b < c->B; b++)
        if (adapter_ids[b] < -1 || adapter_ids[b] >= m->lora_n)
            return sd_fail(SD_EINVAL, "sd_ctx_set_adapters: adapter id outside [-1, n_adapters)");
    SD_HIP(hipDeviceSynchronize());
    SD_HIP(hipMemcpy(c->d_adapter + (size_t)slot * c->B, adapter_ids, sizeof(int32_t) * c->B, hipMemcpyHostToDevice));
    return SD_OK;
}

extern "C" int sd_ctx_attach(sd_ctx *c, sd_model *m)
{
    if (!c || !m) return sd_fail(SD_EINVAL, "sd_ctx_attach: null argument");
    if (find_slot(c, m) >= 0) return SD_OK;
    if (c->n_slots >= SD_MAX_SLOTS) return sd_fail(SD_ECAP, "sd_ctx_attach: too many models");
    size_t bytes = (size_t)m->cfg.n_layers * m->cfg.d_model * c->total_cap * m->esz;
    void *k = nullptr, *v = nullptr;
    hipError_t e = hipMalloc(&k, bytes);
    if (e == hipSuccess) e = hipMalloc(&v, bytes);
    if (e != hipSuccess) {
        if (k) (void)hipFree(k);
        return sd_fail(SD_EHIP, std::string("sd_ctx_attach: hipMalloc KV cache: ") + hipGetErrorString(e));
    }
    // zero-fill so that never-written rows hold finite values
    SD_HIP(hipMemset(k, 0, bytes));
    SD_HIP(hipMemset(v, 0, bytes));
    SD_HIP(hipDeviceSynchronize());
    int s = c->n_slots++;
    c->models[s] = m;
    c->kcache[s] = k;
    c->vcache[s] = v;
    return SD_OK;
}

extern "C" int sd_ctx_set_tokens(sd_ctx *c, const int32_t *tokens, const int32_t *lens, const int32_t *seq_ids,
                                 int32_t n_seq)
{
    if (!c || !tokens || !lens || n_seq < 1 || n_seq > c->B) return sd_fail(SD_EINVAL, "sd_ctx_set_tokens: bad argument");
    SD_HIP(hipDeviceSynchronize());
    size_t pos = 0;
    std::vector<int32_t> zero(SD_MAX_SLOTS, 0);
    for (int j = 0; j < n_seq; j++) {
        int b = seq_ids ? seq_ids[j] : j;
        if (b < 0 || b >= c->B) return sd_fail(SD_EINVAL, "sd_ctx_set_tokens: sequence id out of range");
        if (lens[j] < 1 || lens[j] > c->cap[b]) return sd_fail(SD_ECAP, "sd_ctx_set_tokens: length beyond capacity");
        SD_HIP(hipMemcpy(c->d_tokens + c->off[b], tokens + pos, sizeof(int32_t) * lens[j], hipMemcpyHostToDevice));
        SD_HIP(hipMemcpy(c->d_ntok + b, &lens[j], sizeof(int32_t), hipMemcpyHostToDevice));
        for (int s = 0; s < SD_MAX_SLOTS; s++)
            SD_HIP(hipMemcpy(c->d_kvlen + (size_t)s * c->B + b, &zero[0], sizeof(int32_t), hipMemcpyHostToDevice));
        for (int h = 0; h < 2; h++) // a new sequence starts without acceptance history
            SD_HIP(hipMemcpy(c->d_policy + (size_t)h * c->B + b, &zero[0], sizeof(int32_t), hipMemcpyHostToDevice));
        pos += lens[j];
        c->len_upper = std::max(c->len_upper, lens[j]);
    }
    SD_HIP(hipDeviceSynchronize());
    return SD_OK;
}

extern "C" int sd_ctx_sync(sd_ctx *c, sd_model *m, int32_t *n_tokens, int32_t *kv_len)
{
    if (!c) return sd_fail(SD_EINVAL, "sd_ctx_sync: null context");
    SD_HIP(hipDeviceSynchronize());
    std::vector<int32_t> nt(c->B);
    SD_HIP(hipMemcpy(nt.data(), c->d_ntok, sizeof(int32_t) * c->B, hipMemcpyDeviceToHost));
    c->len_upper = *std::max_element(nt.begin(), nt.end());
    if (n_tokens) memcpy(n_tokens, nt.data(), sizeof(int32_t) * c->B);
    if (m && kv_len) {
        int s = find_slot(c, m);
        if (s < 0) return sd_fail(SD_EINVAL, "sd_ctx_sync: model not attached");
        SD_HIP(hipMemcpy(kv_len, c->d_kvlen + (size_t)s * c->B, sizeof(int32_t) * c->B, hipMemcpyDeviceToHost));
    }
    int32_t st = 0;
    SD_HIP(hipMemcpy(&st, c->d_status, sizeof(int32_t), hipMemcpyDeviceToHost));
    if (st) {
        SD_HIP(hipMemset(c->d_status, 0, sizeof(int32_t)));
        std::string msg = "device status:";
        if (st & 1) msg += " capacity exceeded;";
        if (st & 2) msg += " verify on a sequence whose cache is not at n-1;";
        if (st & 4) msg += " sequence id out of range;";
        if (st & 8) msg += " position beyond the rotary table;";
        if (st & 16) msg += " token id outside the vocabulary;";
        if (st & 32) msg += " cache length beyond the bound the attention launch was sized for;";
        if (st & 64) msg += " draft cache more than two tokens behind its sequence (prefill it first);";
        return sd_fail(SD_ESTATE, msg);
    }
    return SD_OK;
}

extern "C" int sd_ctx_get_tokens(sd_ctx *c, int32_t seq, int32_t *out, int32_t max_tokens, int32_t *n_out)
{
    if (!c || seq < 0 || seq >= c->B || !out || max_tokens < 0) return sd_fail(SD_EINVAL, "sd_ctx_get_tokens: bad argument");
    SD_HIP(hipDeviceSynchronize());
    int32_t n = 0;
    SD_HIP(hipMemcpy(&n, c->d_ntok + seq, sizeof(int32_t), hipMemcpyDeviceToHost));
    int32_t k = std::min(n, max_tokens);
    if (k > 0) SD_HIP(hipMemcpy(out, c->d_tokens + c->off[seq], sizeof(int32_t) * k, hipMemcpyDeviceToHost));
    if (n_out) *n_out = n;
    return SD_OK;
}

extern "C" int sd_ctx_set_kv(sd_ctx *c, sd_model *m, int32_t layer, int32_t seq, const void *k, const void *v,
                             int32_t len)
{
    if (!c || !m || !k || !v) return sd_fail(SD_EINVAL, "sd_ctx_set_kv: null argument");
    int s = find_slot(c, m);
    if (s < 0) return sd_fail(SD_EINVAL, "sd_ctx_set_kv: model not attached");
    if (layer < 0 || layer >= m->cfg.n_layers || seq < 0 || seq >= c->B) return sd_fail(SD_EINVAL, "sd_ctx_set_kv: bad index");
    if (len < 0 || len > c->cap[seq]) return sd_fail(SD_ECAP, "sd_ctx_set_kv: length beyond capacity");
    size_t bytes = (size_t)len * m->cfg.d_model * m->esz;
    void *dk = nullptr, *dv = nullptr;
    if (len > 0) {
        SD_HIP(hipMalloc(&dk, bytes));
        SD_HIP(hipMalloc(&dv, bytes));
        SD_HIP(hipMemcpy(dk, k, bytes, hipMemcpyDefault)); // host or device source
        SD_HIP(hipMemcpy(dv, v, bytes, hipMemcpyDefault));
        size_t lstride = (size_t)m->cfg.d_model * c->total_cap * m->esz;
        hipError_t e = launch_set_kv(0, m->cfg.dtype, dk, dv, len, m->cfg.n_heads, m->cfg.head_dim, c->off[seq],
                                     c->total_cap, (char *)c->kcache[s] + layer * lstride,
                                     (char *)c->vcache[s] + layer * lstride);
        hipError_t e2 = hipDeviceSynchronize();
        (void)hipFree(dk);
        (void)hipFree(dv);
        SD_HIP(e);
        SD_HIP(e2);
    }
    SD_HIP(hipMemcpy(c->d_kvlen + (size_t)s * c->B + seq, &len, sizeof(int32_t), hipMemcpyHostToDevice));
    return SD_OK;
}

extern "C" int sd_ctx_truncate(sd_ctx *c, sd_model *m, int32_t seq, int32_t len)
{
    if (!c || !m || seq < 0 || seq >= c->B || len < 0) return sd_fail(SD_EINVAL, "sd_ctx_truncate: bad argument");
    int s = find_slot(c, m);
    if (s < 0) return sd_fail(SD_EINVAL, "sd_ctx_truncate: model not attached");
    SD_HIP(hipDeviceSynchronize());
    int32_t cur = 0;
    SD_HIP(hipMemcpy(&cur, c->d_kvlen + (size_t)s * c->B + seq, sizeof(int32_t), hipMemcpyDeviceToHost));
    if (len < cur) SD_HIP(hipMemcpy(c->d_kvlen + (size_t)s * c->B + seq, &len, sizeof(int32_t), hipMemcpyHostToDevice));
    return SD_OK;
}

extern "C" int sd_debug_gemm_plan(int32_t mode, int32_t m, int32_t n, int32_t k, int32_t n_per_seg, int32_t plan[6])
{
    if (!plan || m < 1 || n < 1 || k < 1 || n_per_seg < 1) return sd_fail(SD_EINVAL, "sd_debug_gemm_plan: bad argument");
    int p[6];
    if (gemm_tile_plan(mode, m, n, k, n_per_seg, p) != 0)
        return sd_fail(SD_EINVAL, "sd_debug_gemm_plan: not a shape of the row-blocked kernel");
    for (int i = 0; i < 6; i++) plan[i] = p[i];
    return SD_OK;
}

extern "C" int64_t sd_debug_layout_index(int32_t kind, int64_t a, int64_t b, int64_t c, int64_t d)
{
    if (a < 0 || b < 0 || c <= 0) return -1;
    if (kind == 0) return (c % 128 == 0 && b < c && a < ((int64_t)1 << 30)) ? (int64_t)tiled_index((int)a, (int)b, (int)c) : -1;
    if (kind == 1) {
        if (c % 128 != 0 || b >= c || d <= 0 || a >= d) return -1;
        const ActView av = {0, (int32_t)d, 1};
        return (int64_t)act_index(av, (int)a, (int)b, (int)c);
    }
    if (kind == 2) return b < c ? (int64_t)vt_offset((int)c, a, (int)b) : -1;
    if (kind == 3) return (b < c && c % 8 == 0) ? (int64_t)kt_offset((int)c, a, (int)b) : -1;
    return -1;
}

// Test hook: copy one workspace buffer of the last forward to the host as fp32.
// name: "x" [rows][d], "qkv" [rows][3d], "q"/"o"/"a" [rows][d] (hi + lo summed), "act" [rows][d_ffn];
// "seq_order" / "seq_len" [rows]: the last plan's block order and cache lengths (rows = sequences).
extern "C" int sd_debug_read(sd_model *m, const char *name, float *out_host, int32_t rows)
{
    if (!m || !name || !out_host || rows < 0 || rows > m->cfg.max_rows) return sd_fail(SD_EINVAL, "sd_debug_read: bad argument");
    SD_HIP(hipDeviceSynchronize());
    const size_t d = m->cfg.d_model, F = m->cfg.d_ffn;
    if (!strcmp(name, "x") || !strcmp(name, "qkv")) {
        size_t w = !strcmp(name, "x") ? d : 3 * d;
        SD_HIP(hipMemcpy(out_host, !strcmp(name, "x") ? m->x : m->qkv, rows * w * 4, hipMemcpyDeviceToHost));
        return SD_OK;
    }
    if (!strcmp(name, "seq_order") || !strcmp(name, "seq_len")) { // per sequence slot of the last plan, as floats
        std::vector<int32_t> a(rows), b(rows);
        const bool order = !strcmp(name, "seq_order");
        SD_HIP(hipMemcpy(a.data(), order ? m->plan.seq_order : m->plan.seq_kv0, rows * 4, hipMemcpyDeviceToHost));
        SD_HIP(hipMemcpy(b.data(), m->plan.seq_nq, rows * 4, hipMemcpyDeviceToHost));
        for (int r = 0; r < rows; r++) out_host[r] = order ? (float)a[r] : (float)(b[r] > 0 ? a[r] + b[r] : 0);
        return SD_OK;
    }
    const void *src = nullptr;
    size_t w = d, plane = m->plane_d;
    if (!strcmp(name, "q")) src = m->qbuf;
    else if (!strcmp(name, "o")) src = m->obuf;
    else if (!strcmp(name, "a")) src = m->abuf;
    else if (!strcmp(name, "act")) src = m->act, w = F, plane = m->plane_f;
    else return sd_fail(SD_EINVAL, "sd_debug_read: unknown buffer");
    if (m->cfg.dtype == SD_FP32) {
        SD_HIP(hipMemcpy(out_host, src, rows * w * 4, hipMemcpyDeviceToHost));
        return SD_OK;
    }
    // the buffer is laid out for the row count of the forward that wrote it
    const int frows = !strcmp(name, "a") ? m->last_a_rows : m->last_rows;
    if (rows > frows) return sd_fail(SD_EINVAL, "sd_debug_read: more rows than the last forward wrote");
    const ActView av = {plane, frows, (int32_t)(w % 128 == 0)};
    const size_t n = (size_t)frows * w;
    std::vector<uint16_t> hi(n), lo(n);
    SD_HIP(hipMemcpy(hi.data(), src, n * 2, hipMemcpyDeviceToHost));
    SD_HIP(hipMemcpy(lo.data(), (const uint16_t *)src + plane, n * 2, hipMemcpyDeviceToHost));
    for (int r = 0; r < rows; r++)
        for (size_t k = 0; k < w; k++) {
            const size_t i = act_index(av, r, (int)k, (int)w);
            uint32_t a = (uint32_t)hi[i] << 16, b = (uint32_t)lo[i] << 16;
            float fa, fb;
            memcpy(&fa, &a, 4);
            memcpy(&fb, &b, 4);
            out_host[(size_t)r * w + k] = fa + fb;
        }
    return SD_OK;
}

extern "C" int sd_last_logits(sd_model *m, float *out, int32_t max_rows, int32_t *rows)
{
    if (!m || !out || max_rows < 0) return sd_fail(SD_EINVAL, "sd_last_logits: bad argument");
    SD_HIP(hipDeviceSynchronize());
    int n = std::min(m->last_lm_rows, max_rows);
    if (n > 0) SD_HIP(hipMemcpy(out, m->logits, (size_t)n * m->cfg.vocab * sizeof(float), hipMemcpyDeviceToDevice));
    if (rows) *rows = n;
    return SD_OK;
}

// ---------------------------------------------------------------- one decoder forward
static hipError_t gemm_generic(sd_model *m, hipStream_t s, int mode, const void *A, ActView a_av, WeightSeg w, int M,
                               int N, int K, float *C, void *Cact, ActView c_av)
{
    return launch_gemm_generic(s, m->cfg.dtype, mode, A, a_av, w, M, N, K, C, Cact, c_av);
}

// Weight-streaming path for a GEMM whose fp32 result is consumed as split-K slabs.  Returns the number
// of slabs written to `slabs` (slab stride M*N floats), 0 if the shape is outside the kernel's domain.
static const NormFold kNoFold = {nullptr, 0, 0.f, nullptr, nullptr, nullptr, nullptr};
static int stream_gemm(sd_model *m, hipStream_t s, const void *A, ActView a_av, WeightSeg w, int M, int N, int K,
                       float *slabs, size_t slabs_floats, int force_splits, hipError_t *err, int extra_slabs = 0,
                       LmStats ls = {nullptr, 0.f}, int *ls_done = nullptr, NormFold nf = kNoFold)
{
    if (ls_done) *ls_done = 0;
    *err = hipSuccess;
    if (m->cfg.dtype != SD_BF16 || (g_force_generic & 1)) return 0;
    int ns = force_splits > 0 ? force_splits : gemm_skinny_splits(GEMM_STORE, M, N, K, w.n_per_seg);
    // (extra_slabs: slabs the caller appends after the GEMM's own, e.g. a low-rank update)
    if ((size_t)(ns + extra_slabs) * M * N > slabs_floats || ns + extra_slabs > 8) ns = 1;
    if ((size_t)(ns + extra_slabs) * M * N > slabs_floats) return 0;
    const ActView none = {0, 0, 0};
    hipError_t e = launch_gemm_skinny_bf16(s, GEMM_STORE, A, a_av, w, M, N, K, slabs, (size_t)M * N, ns, nullptr, none,
                                           ls, ls_done, nf);
    if (e == hipErrorNotSupported) return 0;
    *err = e;
    return ns;
}

#define FWD(expr)                                                                                  \
    do {                                                                                           \
        hipError_t e__ = (expr);                                                                   \
        if (e__ != hipSuccess)                                                                     \
            return sd_fail(SD_EHIP, std::string("forward: ") + #expr + ": " + hipGetErrorString(e__)); \
    } while (0)

// Rows are laid out as R slots per selected sequence.  Logits are produced for
// n_lm rows (every row for verify, the last valid row of each sequence for
// draft, none when want_logits is false).
//
// Launch schedule per layer (bf16, few rows): [add+]rmsnorm -> QKV GEMM (split-K slabs) -> RoPE + cache
// append (adds the slabs) -> attention -> O GEMM (slabs) -> add + rmsnorm -> gate/up GEMM with SwiGLU
// epilogue -> down GEMM (slabs, added by the next layer's add + rmsnorm).  Shapes outside the MFMA
// kernels' domain, and fp32 models, take the reference kernels with the same data flow.
// One forward over R rows for each of n_seq sequences - or, for prefill (mode PLAN_CATCHUP, G > 1), over G
// groups of R rows per sequence, each group a plan slot of its own.
static int forward(sd_model *m, sd_ctx *c, int slot, hipStream_t s, int mode, int R, int n_seq,
                   const int32_t *seq_ids, int upto_off, const int32_t *cand, int gamma, int cand_idx,
                   bool want_logits, int G = 1, bool plan_ready = false, bool embed_ready = false,
                   float lm_invT = -1.f)
{
    // plan_ready / embed_ready: the draft sampler of the previous token has laid out this single-row forward /
    // has also gathered and normed its rows.  lm_invT >= 0: leave the LM head's per-block softmax partials
    // (1 / temperature, 0 for greedy) for the sampler that follows, where the LM-head kernel can.
    const sd_model_config &cf = m->cfg;
    const int n_slots = n_seq * G; // plan slots: what the attention kernels see as sequences
    const int M = n_slots * R, d = cf.d_model, H = cf.n_heads, hd = cf.head_dim, F = cf.d_ffn, V = cf.vocab;
    if (G < 1 || (G > 1 && mode != PLAN_CATCHUP)) return sd_fail(SD_EINVAL, "forward: row groups are for prefill only");
    if (M > cf.max_rows) return sd_fail(SD_ECAP, "forward: rows exceed the model's max_rows");
    // activation buffers of bf16 models are step-major when their width allows it
    const int sm_d = cf.dtype == SD_BF16 && d % 128 == 0, sm_f = cf.dtype == SD_BF16 && F % 128 == 0;
    const ActView avd = {m->plane_d, M, sm_d}, avf = {m->plane_f, M, sm_f}, av0 = {0, 0, 0};
    m->last_rows = M;
    m->last_a_rows = M;
    CtxView cv = c->view();
    PlanView pv = m->plan;
    int kv_upper = std::min(c->len_upper + SD_MAX_GAMMA + 1, c->max_cap);
    size_t lstride = (size_t)d * c->total_cap * m->esz;
    hipError_t ge;
    // Few rows (the verify pass of a few sequences, draft tokens): the two add + RMSNorm launches of a layer are
    // split between the projection before them and the GEMM after them (NormFold) - seven dependent launches
    // per layer become five.  Needs every GEMM of the forward on the few-row kernels.
    const bool fold = cf.dtype == SD_BF16 && !(g_force_generic & (1 | 16)) && g_norm_fold != 2 && G == 1 && M <= 32 &&
                      m->lora_n == 0 && m->tiled_dd && m->tiled_fd && m->tiled_df && (!want_logits || m->tiled_lm) &&
                      d % 128 == 0 && F % 128 == 0 && V % 16 == 0 && d / 16 <= SD_NORMFOLD_MAX_BLOCKS &&
                      cf.n_layers >= 1;
    const int fold_nb = gemm_normfold_blocks(d);
    const NormFold nf_consume = {m->ss_part, fold_nb, cf.rms_eps, nullptr, nullptr, nullptr, nullptr};
    bool a_scaled = false; // abuf holds rows scaled by the gains only; their sums of squares are in ss_part
    if (!plan_ready) { ProfScope ps(T_PLAN, s); // (the draft sampler lays out the single-row forwards that follow it)
    if (G > 1) FWD(launch_plan_prefill(s, R, G, n_seq, seq_ids, cv, slot, upto_off, V, pv));
    else FWD(launch_plan(s, mode, R, n_seq, seq_ids, cv, slot, upto_off, cand, gamma, cand_idx, V, pv)); }
    if (!embed_ready) { ProfScope ps(T_EMBED, s); // embedding gather + the first layer's norm in one launch
    FWD(launch_embed_rmsnorm(s, cf.dtype, m->embed, pv.row_tok, M, d, m->x, m->norm_attn[0], cf.rms_eps, m->abuf, avd)); }
    int pending = 0; // split-K slabs of the previous down projection not yet added to x
    for (int l = 0; l < cf.n_layers; l++) {
        void *Kl = (char *)c->kcache[slot] + l * lstride, *Vtl = (char *)c->vcache[slot] + l * lstride;
        if (l > 0 && !fold) { ProfScope ps(T_RMSNORM, s);
        if (pending)
            FWD(launch_add_rmsnorm(s, cf.dtype, m->x, m->gpart_r, pending, (size_t)M * d, m->norm_attn[l], nullptr, M, d,
                                   cf.rms_eps, m->abuf, avd));
        else
            FWD(launch_rmsnorm(s, cf.dtype, m->x, m->norm_attn[l], nullptr, M, d, cf.rms_eps, m->abuf, avd));
        }
        pending = 0;
        WeightSeg wqkv = {{m->wq[l], m->wk[l], m->wv[l]}, d, m->tiled_dd, m->stream_nt};
        int nq_slabs;
        const float *qkv_src;
        // low-rank adapters (sequences of one batch may use different ones): their update of q, k, v is one more
        // slab for the consumer to add - or is added in place where the GEMM left a single full result
        const bool lora_qkv = m->lora_n > 0 && (m->lora_a[0][l] || m->lora_a[1][l] || m->lora_a[2][l]);
        const bool lora_o = m->lora_n > 0 && m->lora_a[3][l];
        bool qkv_in_place = false;
        { ProfScope ps(T_QKV, s);
        nq_slabs = stream_gemm(m, s, m->abuf, avd, wqkv, M, 3 * d, d, m->gpart_q, m->gpart_q_floats, 0, &ge, lora_qkv ? 1 : 0,
                               LmStats{nullptr, 0.f}, nullptr, a_scaled ? nf_consume : kNoFold);
        FWD(ge);
        qkv_src = m->gpart_q;
        if (!nq_slabs && fold) return sd_fail(SD_EHIP, "forward: QKV shape left the few-row kernels under the split norm");
        if (!nq_slabs) {
            FWD(gemm_generic(m, s, GEMM_STORE, m->abuf, avd, wqkv, M, 3 * d, d, m->qkv, nullptr, av0));
            nq_slabs = 1;
            qkv_src = m->qkv;
            qkv_in_place = true;
        } }
        if (lora_qkv) { ProfScope ps(T_LORA, s);
            const float *A3[3] = {m->lora_a[0][l], m->lora_a[1][l], m->lora_a[2][l]};
            const float *B3[3] = {m->lora_b[0][l], m->lora_b[1][l], m->lora_b[2][l]};
            float *dst = qkv_in_place ? m->qkv : m->gpart_q + (size_t)nq_slabs * M * 3 * d;
            FWD(launch_lora_delta(s, cf.dtype, m->abuf, avd, M, d, d, 3, pv, cv.adapter + (size_t)slot * cv.B, m->lora_n,
                                  m->lora_rank, m->lora_scale, A3, B3, dst, qkv_in_place ? 1 : 0));
            if (!qkv_in_place) nq_slabs++;
        }
        hipError_t ea = hipErrorNotSupported;
        int oproj_done = 0; // the attention blocks applied the output projection themselves: H slabs in gpart_r
        // RoPE + append + attention in one launch - unless a sequence spans several slots (prefill): their
        // rows must all be in the cache before any slot's attention starts
        if (cf.dtype == SD_BF16 && !(g_force_generic & 2) && G == 1) {
            ProfScope ps(T_ATTN, s);
            const bool try_oproj = !fold && !lora_o && m->tiled_dd && !(g_force_generic & (1 | 8));
            ea = launch_attn_fused_bf16(s, qkv_src, nq_slabs, (size_t)M * 3 * d, pv, cv, R, n_seq, H, hd, m->rope,
                                        cf.max_pos, Kl, Vtl, c->total_cap, kv_upper, m->obuf, avd, m->stream_nt,
                                        try_oproj ? m->wo[l] : nullptr, d, m->gpart_r, m->gpart_r_floats, &oproj_done);
        }
        if (ea == hipErrorNotSupported) {
            { ProfScope ps(T_ROPE, s);
            FWD(launch_rope_append(s, cf.dtype, qkv_src, nq_slabs, (size_t)M * 3 * d, pv, cv, M, R, H, hd, m->rope,
                                   cf.max_pos, m->qbuf, avd, Kl, Vtl, c->total_cap)); }
            ProfScope ps(T_ATTN, s);
            if (cf.dtype == SD_BF16 && !(g_force_generic & 2) && G > 1) // a prompt's row groups share their K / V tiles
                ea = launch_attn_prefill_bf16(s, m->qbuf, avd, Kl, Vtl, pv, cv, R, n_seq, G, H, hd, c->total_cap, kv_upper,
                                              m->part, m->part_floats, m->obuf, avd);
            if (ea == hipErrorNotSupported && cf.dtype == SD_BF16 && !(g_force_generic & 2))
                ea = launch_attn_mfma_bf16(s, m->qbuf, avd, Kl, Vtl, pv, cv, R, n_slots, H, hd, c->total_cap,
                                           kv_upper, m->part, m->part_floats, m->obuf, avd,
                                           m->stream_nt && G == 1); // (the row groups of a prefill re-read one prefix: let it stay cached)
            if (ea == hipErrorNotSupported)
                // (its score buffer is sized from the largest capacity, which never changes: a captured graph
                // stays valid however far the sequences have grown since the capture)
                ea = launch_attn_generic(s, cf.dtype, m->qbuf, avd, Kl, Vtl, pv, cv, R, n_slots, H, hd,
                                         c->total_cap, c->max_cap, m->obuf, avd);
        }
        if (ea == hipErrorNotSupported) return sd_fail(SD_ECAP, "forward: context too long for the generic attention kernel");
        FWD(ea);
        WeightSeg wo = {{m->wo[l], nullptr, nullptr}, d, m->tiled_dd, m->stream_nt};
        int no_slabs = H;
        if (fold) { ProfScope ps(T_OPROJ, s); // projection + residual + the gains of the norm that follows
            const NormFold nf_p = {nullptr, 0, 0.f, m->x, m->norm_ffn[l], m->ss_part, nullptr};
            const hipError_t eo = launch_gemm_skinny_bf16(s, GEMM_STORE, m->obuf, avd, wo, M, d, d, nullptr, 0, 1, m->abuf, avd,
                                                          LmStats{nullptr, 0.f}, nullptr, nf_p);
            FWD(eo);
            a_scaled = true;
        } else if (!oproj_done) { ProfScope ps(T_OPROJ, s);
        no_slabs = stream_gemm(m, s, m->obuf, avd, wo, M, d, d, m->gpart_r, m->gpart_r_floats, 0, &ge, lora_o ? 1 : 0);
        FWD(ge);
        if (!no_slabs) FWD(gemm_generic(m, s, GEMM_RESID, m->obuf, avd, wo, M, d, d, m->x, nullptr, av0)); }
        if (lora_o) { ProfScope ps(T_LORA, s); // (without slabs the projection was added to x directly: so is its update)
            const float *A1[1] = {m->lora_a[3][l]}, *B1[1] = {m->lora_b[3][l]};
            float *dst = no_slabs ? m->gpart_r + (size_t)no_slabs * M * d : m->x;
            FWD(launch_lora_delta(s, cf.dtype, m->obuf, avd, M, d, d, 1, pv, cv.adapter + (size_t)slot * cv.B, m->lora_n,
                                  m->lora_rank, m->lora_scale, A1, B1, dst, no_slabs ? 0 : 1));
            if (no_slabs) no_slabs++;
        }
        if (!fold) { ProfScope ps(T_RMSNORM, s);
        if (no_slabs)
            FWD(launch_add_rmsnorm(s, cf.dtype, m->x, m->gpart_r, no_slabs, (size_t)M * d, m->norm_ffn[l], nullptr, M, d,
                                   cf.rms_eps, m->abuf, avd));
        else
            FWD(launch_rmsnorm(s, cf.dtype, m->x, m->norm_ffn[l], nullptr, M, d, cf.rms_eps, m->abuf, avd));
        }
        WeightSeg wgu = {{m->wgate[l], m->wup[l], nullptr}, F, m->tiled_fd, m->stream_nt};
        { ProfScope ps(T_GATEUP, s);
        hipError_t eg = hipErrorNotSupported;
        if (cf.dtype == SD_BF16 && !(g_force_generic & 1))
            eg = launch_gemm_skinny_bf16(s, GEMM_SWIGLU, m->abuf, avd, wgu, M, F, d, nullptr, 0, 1, m->act,
                                         avf, LmStats{nullptr, 0.f}, nullptr, a_scaled ? nf_consume : kNoFold);
        if (eg == hipErrorNotSupported && fold)
            return sd_fail(SD_EHIP, "forward: gate/up shape left the few-row kernels under the split norm");
        if (eg == hipErrorNotSupported)
            eg = gemm_generic(m, s, GEMM_SWIGLU, m->abuf, avd, wgu, M, F, d, nullptr, m->act, avf);
        FWD(eg); }
        WeightSeg wd = {{m->wdown[l], nullptr, nullptr}, d, m->tiled_df, m->stream_nt};
        if (fold) { ProfScope ps(T_DOWN, s); // projection + residual + the gains of the next layer's (or the final) norm
            const float *g_next = l + 1 < cf.n_layers ? m->norm_attn[l + 1] : m->final_norm;
            const NormFold nf_p = {nullptr, 0, 0.f, m->x, g_next, m->ss_part, nullptr};
            const hipError_t ed = launch_gemm_skinny_bf16(s, GEMM_STORE, m->act, avf, wd, M, d, F, nullptr, 0, 1, m->abuf, avd,
                                                          LmStats{nullptr, 0.f}, nullptr, nf_p);
            FWD(ed);
            pending = 0;
        } else { ProfScope ps(T_DOWN, s);
        pending = stream_gemm(m, s, m->act, avf, wd, M, d, F, m->gpart_r, m->gpart_r_floats, 0, &ge);
        FWD(ge);
        if (!pending) FWD(gemm_generic(m, s, GEMM_RESID, m->act, avf, wd, M, d, F, m->x, nullptr, av0)); }
    }
    if (want_logits) {
        int n_lm = mode == PLAN_VERIFY ? M : n_seq;
        const ActView avlm = fold ? avd : ActView{m->plane_d, n_lm, sm_d}; // (split norm: the rows stay where the last down projection put them)
        m->last_a_rows = fold ? M : n_lm;
        if (!fold) { ProfScope ps(T_RMSNORM, s);
        if (pending)
            FWD(launch_add_rmsnorm(s, cf.dtype, m->x, m->gpart_r, pending, (size_t)M * d, m->final_norm, pv.lm_row, n_lm,
                                   d, cf.rms_eps, m->abuf, avlm));
        else
            FWD(launch_rmsnorm(s, cf.dtype, m->x, m->final_norm, pv.lm_row, n_lm, d, cf.rms_eps, m->abuf, avlm));
        }
        WeightSeg wl = {{m->lm_head, nullptr, nullptr}, V, m->tiled_lm, m->stream_nt};
        { ProfScope ps(T_LMHEAD, s);
        const LmStats ls = {lm_invT >= 0.f && V % 32 == 0 ? m->lm_stats : nullptr, lm_invT >= 0.f ? lm_invT : 0.f};
        int ls_done = 0;
        NormFold nf_lm = kNoFold;
        if (fold) { // (a_scaled: there is at least one layer)
            nf_lm = nf_consume;
            nf_lm.row_map = pv.lm_row;
        }
        int nl = stream_gemm(m, s, m->abuf, avlm, wl, n_lm, V, d, m->logits, (size_t)cf.max_rows * V, 1, &ge, 0, ls, &ls_done, nf_lm);
        FWD(ge);
        if (!nl && fold) return sd_fail(SD_EHIP, "forward: LM head shape left the few-row kernels under the split norm");
        m->lm_stats_nb = nl && ls_done ? V / 32 : 0;
        if (!nl) FWD(gemm_generic(m, s, GEMM_STORE, m->abuf, avlm, wl, n_lm, V, d, m->logits, nullptr, av0)); }
        m->last_lm_rows = n_lm;
    }
    return SD_OK;
}

static int check_call(const char *who, sd_model *m, sd_ctx *c, int n_seq, int *slot)
{
    if (!m || !c) return sd_fail(SD_EINVAL, std::string(who) + ": null model or context");
    if (n_seq < 1 || n_seq > c->B) return sd_fail(SD_EINVAL, std::string(who) + ": n_seq out of range");
    *slot = find_slot(c, m);
    if (*slot < 0) return sd_fail(SD_EINVAL, std::string(who) + ": model not attached to this context");
    return SD_OK;
}

extern "C" int sd_prefill(sd_model *m, sd_ctx *c, const int32_t *seq_ids, int32_t n_seq, int32_t max_new,
                          void *stream)
{
    int slot;
    int rc = check_call("sd_prefill", m, c, n_seq, &slot);
    if (rc) return rc;
    if (max_new < 0) return sd_fail(SD_EINVAL, "sd_prefill: max_new < 0");
    int R = std::min(m->cfg.max_rows / n_seq, 16);
    if (R < 1) return sd_fail(SD_ECAP, "sd_prefill: n_seq exceeds the model's max_rows");
    // as many 16-row groups per sequence and forward as the workspace holds: the GEMMs then run at
    // M = n_seq * 16 * G rows and stream the weights once per 16 * G tokens instead of once per 16
    int G = R == 16 ? std::max(1, std::min(m->cfg.max_rows / (16 * n_seq), (max_new + 15) / 16)) : 1;
    for (int done = 0; done < max_new; done += R * G) {
        rc = forward(m, c, slot, (hipStream_t)stream, PLAN_CATCHUP, R, n_seq, seq_ids, 1, nullptr, 0, 0, false, G);
        if (rc) return rc;
    }
    return SD_OK;
}

extern "C" int sd_draft(sd_model *draft, sd_ctx *c, const int32_t *seq_ids, int32_t n_seq, int32_t gamma,
                        float temperature, const float *uniforms, int32_t *cand, float *q, void *stream)
{
    int slot;
    int rc = check_call("sd_draft", draft, c, n_seq, &slot);
    if (rc) return rc;
    if (gamma < 1 || gamma > SD_MAX_GAMMA) return sd_fail(SD_ECAP, "sd_draft: gamma must be in [1, 15]");
    if (!cand) return sd_fail(SD_EINVAL, "sd_draft: null cand");
    if (!(temperature >= 0.f)) return sd_fail(SD_EINVAL, "sd_draft: negative temperature");
    if (temperature > 0.f && (!uniforms || !q)) return sd_fail(SD_EINVAL, "sd_draft: sampling needs uniforms and q");
    if (2 * n_seq > draft->cfg.max_rows) return sd_fail(SD_ECAP, "sd_draft: 2*n_seq exceeds the model's max_rows");
    hipStream_t s = (hipStream_t)stream;
    const sd_model_config &cf = draft->cfg;
    const float lm_invT = temperature > 0.f ? 1.0f / temperature : 0.f;
    int embedded = 0; // the previous sampler has run the first step of this forward
    for (int i = 0; i < gamma; i++) {
        if (i == 0) rc = forward(draft, c, slot, s, PLAN_CATCHUP, 2, n_seq, seq_ids, 0, nullptr, gamma, 0, true, 1, false, false, lm_invT);
        else rc = forward(draft, c, slot, s, PLAN_CAND, 1, n_seq, seq_ids, 0, cand, gamma, i - 1, true, 1, true, embedded != 0, lm_invT);
        if (rc) return rc;
        ProfScope ps(T_SAMPLE, s);
        // every sampler but the last also writes the plan of the forward that feeds its token (the last
        // candidate is never fed) - and, where it works from the LM head's partials, runs that forward's
        // first step (its rows: one per sequence)
        NextPlan next = {draft->plan, c->view(), seq_ids, slot, cf.vocab, i + 1 < gamma ? 1 : 0, gamma, i + 1};
        next.embed = cf.dtype == SD_BF16 && !(g_force_generic & 4);
        next.d = cf.d_model;
        next.E = draft->embed;
        next.x = draft->x;
        next.g = draft->norm_attn[0];
        next.eps = cf.rms_eps;
        next.out = draft->abuf;
        next.av = ActView{draft->plane_d, n_seq, cf.dtype == SD_BF16 && cf.d_model % 128 == 0};
        const bool use_stats = draft->lm_stats_nb > 0 && !(g_force_generic & 4);
        hipError_t e = launch_draft_sample(s, draft->logits, n_seq, cf.vocab, temperature, uniforms, gamma, i, cand, q,
                                           next, use_stats ? draft->lm_stats : nullptr, use_stats ? draft->lm_stats_nb : 0,
                                           &embedded);
        if (e != hipSuccess) return sd_fail(SD_EHIP, std::string("sd_draft: sample: ") + hipGetErrorString(e));
    }
    return SD_OK;
}

extern "C" int sd_verify(sd_model *target, sd_ctx *c, const int32_t *seq_ids, int32_t n_seq, int32_t gamma,
                         float temperature, const int32_t *cand, const float *q, const float *uniforms,
                         int32_t *n_accepted, int32_t *next_token, int32_t commit, void *stream)
{
    int slot;
    int rc = check_call("sd_verify", target, c, n_seq, &slot);
    if (rc) return rc;
    if (gamma < 0 || gamma > SD_MAX_GAMMA) return sd_fail(SD_ECAP, "sd_verify: gamma must be in [0, 15]");
    if (!n_accepted || !next_token) return sd_fail(SD_EINVAL, "sd_verify: null output");
    if (gamma > 0 && !cand) return sd_fail(SD_EINVAL, "sd_verify: null cand");
    if (!(temperature >= 0.f)) return sd_fail(SD_EINVAL, "sd_verify: negative temperature");
    if (temperature > 0.f && (!uniforms || (gamma > 0 && !q)))
        return sd_fail(SD_EINVAL, "sd_verify: sampling needs uniforms and q");
    if (n_seq * (gamma + 1) > target->cfg.max_rows) return sd_fail(SD_ECAP, "sd_verify: rows exceed the model's max_rows");
    hipStream_t s = (hipStream_t)stream;
    rc = forward(target, c, slot, s, PLAN_VERIFY, gamma + 1, n_seq, seq_ids, 0, cand, gamma, 0, true);
    if (rc) return rc;
    ProfScope ps(T_TAIL, s);
    hipError_t e = launch_verify_tail(s, target->logits, n_seq, gamma, target->cfg.vocab, temperature, cand, q,
                                      uniforms, seq_ids, n_accepted, next_token, commit, c->view(), target->vstats);
    if (e != hipSuccess) return sd_fail(SD_EHIP, std::string("sd_verify: tail: ") + hipGetErrorString(e));
    if (commit) c->len_upper = std::min(c->len_upper + gamma + 1, c->max_cap);
    return SD_OK;
}

extern "C" int sd_commit(sd_ctx *c, const int32_t *seq_ids, int32_t n_seq, int32_t gamma, const int32_t *cand,
                         const int32_t *n_accepted, const int32_t *next_token, void *stream)
{
    if (!c || !n_accepted || !next_token || (gamma > 0 && !cand)) return sd_fail(SD_EINVAL, "sd_commit: null argument");
    if (n_seq < 1 || n_seq > c->B || gamma < 0 || gamma > SD_MAX_GAMMA) return sd_fail(SD_EINVAL, "sd_commit: bad n_seq or gamma");
    hipError_t e = launch_commit((hipStream_t)stream, c->view(), seq_ids, n_seq, gamma, cand, n_accepted, next_token);
    if (e != hipSuccess) return sd_fail(SD_EHIP, std::string("sd_commit: ") + hipGetErrorString(e));
    c->len_upper = std::min(c->len_upper + gamma + 1, c->max_cap);
    return SD_OK;
}

// ---------------------------------------------------------------- per-sequence candidate counts (Equation 1 in the loop)
extern "C" int sd_policy_set(sd_ctx *c, const int32_t *gammas)
{
    if (!c) return sd_fail(SD_EINVAL, "sd_policy_set: null context");
    SD_HIP(hipDeviceSynchronize());
    if (!gammas) {
        c->use_gamma = 0;
        return SD_OK;
    }
    for (int b = 0; b < c->B; b++)
        if (gammas[b] < 0 || gammas[b] > SD_MAX_GAMMA) return sd_fail(SD_EINVAL, "sd_policy_set: gamma outside [0, 15]");
    SD_HIP(hipMemcpy(c->d_gamma, gammas, sizeof(int32_t) * c->B, hipMemcpyHostToDevice));
    c->use_gamma = 1;
    return SD_OK;
}

extern "C" int sd_policy_choose(sd_ctx *c, const int32_t *seq_ids, int32_t n_seq, double c_ratio, int32_t gamma_max,
                                double alpha0, int32_t *gammas_out, void *stream)
{
    if (!c) return sd_fail(SD_EINVAL, "sd_policy_choose: null context");
    if (n_seq < 1 || n_seq > c->B) return sd_fail(SD_EINVAL, "sd_policy_choose: n_seq out of range");
    if (!(c_ratio >= 0.0) || !(alpha0 >= 0.0 && alpha0 <= 1.0) || gamma_max < 0 || gamma_max > SD_MAX_GAMMA)
        return sd_fail(SD_EINVAL, "sd_policy_choose: c >= 0, alpha0 in [0,1], 0 <= gamma_max <= 15");
    if (!c->use_gamma) { // sequences outside this selection keep the largest count until they are chosen for
        std::vector<int32_t> all(c->B, gamma_max);
        SD_HIP(hipMemcpyAsync(c->d_gamma, all.data(), sizeof(int32_t) * c->B, hipMemcpyHostToDevice, (hipStream_t)stream));
        SD_HIP(hipStreamSynchronize((hipStream_t)stream));
        c->use_gamma = 1;
    }
    hipError_t e = launch_policy_choose((hipStream_t)stream, c->view(), seq_ids, n_seq, c_ratio, gamma_max, alpha0, c->d_gamma,
                                        gammas_out);
    if (e != hipSuccess) return sd_fail(SD_EHIP, std::string("sd_policy_choose: ") + hipGetErrorString(e));
    return SD_OK;
}

extern "C" int sd_policy_read(sd_ctx *c, int32_t *gammas, int32_t *accepted, int32_t *examined)
{
    if (!c) return sd_fail(SD_EINVAL, "sd_policy_read: null context");
    SD_HIP(hipDeviceSynchronize());
    if (gammas) SD_HIP(hipMemcpy(gammas, c->d_gamma, sizeof(int32_t) * c->B, hipMemcpyDeviceToHost));
    if (accepted) SD_HIP(hipMemcpy(accepted, c->d_policy, sizeof(int32_t) * c->B, hipMemcpyDeviceToHost));
    if (examined) SD_HIP(hipMemcpy(examined, c->d_policy + c->B, sizeof(int32_t) * c->B, hipMemcpyDeviceToHost));
    return c->use_gamma ? 1 : 0;
}

extern "C" int sd_debug_stream_read(const void *buf, size_t bytes, uint32_t *scratch_word, void *stream)
{
    if (!buf || !scratch_word || bytes < 16 || ((uintptr_t)buf & 15)) return sd_fail(SD_EINVAL, "sd_debug_stream_read: bad argument");
    hipError_t e = launch_stream_read((hipStream_t)stream, buf, bytes, scratch_word);
    if (e != hipSuccess) return sd_fail(SD_EHIP, std::string("sd_debug_stream_read: ") + hipGetErrorString(e));
    return SD_OK;
}

extern "C" int sd_route(const float *W, const float *b, int32_t n_drafts, int32_t emb_dim, const float *prompt_emb,
                        int32_t n, int32_t *draft_id, void *stream)
{
    if (!W || !prompt_emb || !draft_id) return sd_fail(SD_EINVAL, "sd_route: null argument");
    if (n_drafts < 1 || emb_dim < 1 || n < 1) return sd_fail(SD_EINVAL, "sd_route: non-positive size");
    hipError_t e = launch_route((hipStream_t)stream, W, b, n_drafts, emb_dim, prompt_emb, n, draft_id);
    if (e != hipSuccess) return sd_fail(SD_EHIP, std::string("sd_route: ") + hipGetErrorString(e));
    return SD_OK;
}
