// Internal declarations shared by the HIP sources of libsd (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/sd.h"

#define SD_MAX_SLOTS 8
#define SD_MAX_GAMMA 15
#define SD_ATTN_MAX_SPLITS 32

// ---------------------------------------------------------------- element types
struct bf16_t {
    uint16_t v;
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float((uint32_t)x.v << 16); }

// fp32 -> bf16, round to nearest, ties to even: the hardware conversion (v_cvt_pk_bf16_f32), which gives,
// for every non-NaN fp32 value, the bits of the integer formula  (u + 0x7fff + ((u >> 16) & 1)) >> 16
// (checked exhaustively on the device).
__device__ __forceinline__ uint16_t bf16_bits_rne(float f)
{
    const __bf16 b = (__bf16)f;
    return __builtin_bit_cast(uint16_t, b);
}
// Two values at once: a in the low half, b in the high half of the result.
__device__ __forceinline__ uint32_t bf16x2_bits_rne(float a, float b)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// hi + lo split of two values: hi = bf16(x), lo = bf16(x - hi), both packed like bf16x2_bits_rne.
__device__ __forceinline__ void bf16x2_split(float a, float b, uint32_t &hi, uint32_t &lo)
{
    hi = bf16x2_bits_rne(a, b);
    lo = bf16x2_bits_rne(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}

template <typename T>
__device__ __forceinline__ T from_float(float f);
template <>
__device__ __forceinline__ float from_float<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float f)
{
    bf16_t r;
    r.v = bf16_bits_rne(f);
    return r;
}

// GEMM-input activations.  fp32 models: one fp32 plane.  bf16 models: two bf16
// planes, value = hi + lo with hi = bf16(x), lo = bf16(x - hi), i.e. about 16
// mantissa bits fed to the matrix cores as two operands.  `plane` is the element
// offset from the hi plane to the lo plane.
__device__ __forceinline__ float load_act(const float *b, size_t i, size_t) { return b[i]; }
__device__ __forceinline__ float load_act(const bf16_t *b, size_t i, size_t plane)
{
    return to_float(b[i]) + to_float(b[i + plane]);
}
__device__ __forceinline__ void store_act(float *b, size_t i, size_t, float v) { b[i] = v; }
__device__ __forceinline__ void store_act(bf16_t *b, size_t i, size_t plane, float v)
{
    uint16_t hi = bf16_bits_rne(v);
    b[i].v = hi;
    b[i + plane].v = bf16_bits_rne(v - __uint_as_float((uint32_t)hi << 16));
}

// Four consecutive elements at an index that is a multiple of 4: one 8-byte store per bf16 plane.
__device__ __forceinline__ void store_act4(float *b, size_t i, size_t, float v0, float v1, float v2, float v3)
{
    *(float4 *)(b + i) = make_float4(v0, v1, v2, v3);
}
__device__ __forceinline__ void store_act4(bf16_t *b, size_t i, size_t plane, float v0, float v1, float v2, float v3)
{
    uint32_t h0, l0, h1, l1;
    bf16x2_split(v0, v1, h0, l0);
    bf16x2_split(v2, v3, h1, l1);
    *(uint2 *)(b + i) = make_uint2(h0, h1);
    *(uint2 *)(b + i + plane) = make_uint2(l0, l1);
}

// Where element (row m, column k) of a GEMM-input activation buffer of width K lives.  Row-major, or
// (bf16 buffers whose width is a multiple of 128) "step-major": the 128 columns of K step k/128 of all
// rows of this forward are contiguous, [k/128][m][k%128].  A GEMM block then finds the rows it needs for
// one K step in one contiguous piece instead of at a stride of 2K bytes (which lands on one L2 channel).
// Row-blocked kernels read whole row blocks: activation buffers carry this many rows of slack at the end.
#define SD_ACT_PAD_ROWS 96
struct ActView {
    size_t plane;  // element offset from the hi plane to the lo plane (unused for fp32)
    int32_t rows;  // rows of this forward (the row stride of a step in the step-major order)
    int32_t sm;    // 1 = step-major
};
__host__ __device__ __forceinline__ size_t act_index(ActView v, int m, int k, int K)
{
    return v.sm ? ((size_t)(k >> 7) * v.rows + m) * 128 + (k & 127) : (size_t)m * K + k;
}

// Value cache of one head: 32-token tiles, each stored transposed as [head_dim][32], so that the V^T
// tile a wave multiplies (head_dim x 32 tokens) is one contiguous piece.  t is the row inside the head's
// cache (sequence offset + position; sequence offsets are multiples of 64).
__host__ __device__ __forceinline__ size_t vt_offset(int hd, int64_t t, int d)
{
    return (size_t)(t >> 5) * (size_t)(32 * hd) + (size_t)d * 32 + (size_t)(t & 31);
}

// Key cache of one head: 32-token tiles in the operand order of the score MFMAs.  The scores of a tile
// come from two 16-row operands: operand a holds tokens 8*(i/4) + i%4 in its rows i = 0..15, operand b those
// + 4 (this permutation is what lets the result feed the second product without a shuffle).  Piece
// (c, ab, g, i) - dimensions 32c + 8g .. +8 of the token in row i of operand ab - sits at 16-byte slot
// (2c + ab) * 64 + 16g + i of the tile, so each load instruction of a wave reads one contiguous KiB.
__host__ __device__ __forceinline__ size_t kt_offset(int hd, int64_t t, int d)
{
    const int tok = (int)(t & 31);
    const int ab = (tok >> 2) & 1, i = (tok >> 3) * 4 + (tok & 3);
    const int G = (hd < 32 ? hd : 32) >> 3; // 8-dimension groups per 32-dimension chunk (4 unless head_dim < 32)
    return (size_t)(t >> 5) * (size_t)(32 * hd) + (size_t)(((((d >> 5) * 2 + ab) * G + ((d >> 3) & 3)) * 16 + i) * 8 + (d & 7));
}

// ---------------------------------------------------------------- cross-lane helpers (DPP: the vector ALU's own data path)
template <int CTRL> __device__ __forceinline__ int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); }
template <int CTRL> __device__ __forceinline__ float dpp_f(float v) { return __int_as_float(dpp_i<CTRL>(__float_as_int(v))); }
__device__ __forceinline__ float lane_f(float v, int l) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l)); }
// DPP controls: quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E; row_half_mirror = 0x141; row_mirror = 0x140;
// row_shr:n = 0x110 + n (lanes without a source read 0).
// Sum over each 16-lane row, left in every lane of the row (both sides of each exchange add the same two
// numbers, so all lanes agree bit for bit).
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    v += dpp_f<0x140>(v);
    return v;
}
__device__ __forceinline__ float wave_sum_dpp(float v)
{
    v = row16_sum(v);
    return (lane_f(v, 0) + lane_f(v, 16)) + (lane_f(v, 32) + lane_f(v, 48));
}

// ---------------------------------------------------------------- views passed to kernels
// Device-side view of a context.  kvlen is [SD_MAX_SLOTS][B].
struct CtxView {
    int32_t B;
    int32_t n_slots;
    const int64_t *off; // [B] token / cache-row offset of each sequence
    const int32_t *cap; // [B]
    int32_t *tokens;    // [total_cap]
    int32_t *ntok;      // [B]
    int32_t *kvlen;     // [SD_MAX_SLOTS][B]
    int32_t *status;    // [1] sticky error bits
    const int32_t *adapter; // [SD_MAX_SLOTS][B] low-rank adapter of each sequence per model slot (-1: none)
    const int32_t *gam;     // [B] candidates per step of each sequence, or nullptr: the call's gamma for all
    int32_t *pol;           // [2][B] accepted / examined candidates so far (the running estimate of Equation 1's alpha)
};
// candidates sequence b drafts / has verified in a call made with `gamma` row slots
__device__ __forceinline__ int seq_gamma(const CtxView &cv, int b, int gamma)
{
    if (!cv.gam) return gamma;
    const int g = cv.gam[b];
    return g < 0 ? 0 : (g > gamma ? gamma : g);
}

// Row plan of one forward: R row slots per selected sequence j (rows j*R .. j*R+R-1).
struct PlanView {
    int32_t *row_tok;   // [M] token id fed in this row
    int32_t *row_pos;   // [M] position (= cache row it is appended to)
    int32_t *row_b;     // [M] sequence index in the context
    int32_t *row_valid; // [M] 0 for unused slots
    int32_t *seq_b;     // [n_seq]
    int32_t *seq_kv0;   // [n_seq] cache length before this forward
    int32_t *seq_nq;    // [n_seq] valid rows of this sequence
    int32_t *seq_order; // [n_seq] sequence slots by decreasing cache length: the order attention blocks start in
    int32_t *lm_row;    // [n_lm] source row of each logits row
};

enum PlanMode { PLAN_CATCHUP = 0, PLAN_CAND = 1, PLAN_VERIFY = 2 };

// What the draft sampler needs to lay out the next single-row forward (PLAN_CAND) itself: its block of
// sequence j knows the token just drawn, so it writes that sequence's plan entries and advances the cache
// length, and the forward that follows starts without a plan launch.  enabled = 0: do nothing.
struct NextPlan {
    PlanView pv;
    CtxView cv;
    const int32_t *seq_ids;
    int32_t slot, vocab, enabled;
    int32_t gamma, next_idx; // row slots of the draft call; index of the candidate the planned forward leads to
    // (samplers that run 256-thread blocks only) the planned forward's first step as well: embedding row of the
    // token into x[j] and the first layer's norm of it into the activation buffer, as embed_rmsnorm_kernel does
    int32_t embed; // 0: the forward gathers and norms the row itself
    int32_t d;
    const void *E;  // bf16 [vocab][d]
    float *x;
    const float *g; // first layer's attention-norm gains
    float eps;
    void *out;
    ActView av;
};

struct WeightSeg { // up to three matrices stacked along N (q,k,v or gate,up)
    const void *p[3];
    int32_t n_per_seg;
    int32_t tiled; // 1: every segment is stored in the 16 x 128 tile order below instead of row-major
    int32_t nt;    // 1: the few-row kernels read these weights with the nontemporal hint (see ld_stream)
};

// A load of data that is read once per forward.  With the nontemporal hint a stream that is larger than the
// caches runs measurably faster on this part (a plain read of 1 GiB: 7.0 against 6.1 TB/s; the 180 MB gate/up
// stream of the 7B shape at 6 rows: 31.9 against 35.2 us); data that would have stayed resident in the 256 MB
// memory-side cache between calls (a small draft model's weights) is better read without it.
template <bool NT, typename T>
__device__ __forceinline__ T ld_stream(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

// Tiled weight order (bf16 matrices [N][K] with N % 16 == 0 and K % 128 == 0).  The 4 KiB that one wave
// consumes per 128-element K step - 16 rows x 128 elements - are contiguous, steps of a 16-row tile
// follow each other along K, and inside a step the 16-byte pieces are in MFMA operand order: piece
// (i, g, r) = row r, elements 32*i + 8*g .. +8, at byte offset 1024*i + 16*(16*g + r).  A wave's load
// instruction i therefore reads one contiguous kilobyte (lane = 16*g + r).  Row-major rows of 2*K bytes
// put the 16 rows of such a load at a stride that maps to a single L2 channel, which caps one compute
// unit at ~37 GB/s; the tiled order streams at ~100 GB/s per unit.
#define SD_TILE_ROWS 16
#define SD_TILE_K 128
__host__ __device__ __forceinline__ size_t tiled_index(int n, int k, int K)
{
    const size_t step = (size_t)(n >> 4) * (size_t)(K >> 7) + (size_t)(k >> 7);
    const int kk = k & 127;
    return step * 2048 + (size_t)((kk >> 5) * 512 + ((((kk >> 3) & 3) * 16 + (n & 15)) * 8) + (kk & 7));
}
__host__ __device__ __forceinline__ size_t weight_index(int n, int k, int K, int tiled)
{
    return tiled ? tiled_index(n, k, K) : (size_t)n * K + k;
}

enum GemmMode { GEMM_STORE = 0, GEMM_RESID = 1, GEMM_SWIGLU = 2 };

// RMSNorm split between the GEMM that produces a residual update and the GEMM that consumes the normed rows
// (few-row kernels), so that no launch of its own stands between them.  Producer (GEMM_STORE without K split,
// one block per group of output columns): x[m][n] += result; the operand buffer of the next GEMM receives
// hi + lo of x[m][n] * g[n] - scaled by the gains but not yet by 1 / rms, which needs the whole row - and
// ss_out[m * SD_NORMFOLD_MAX_BLOCKS + block] the block's share of sum_n x[m][n]^2.  Consumer: multiplies row m of
// its sums by 1 / sqrt(sum_b ss_in[m * SD_NORMFOLD_MAX_BLOCKS + b] / K + eps).  The scaling commutes with the product; what moves is the
// point where the operand is rounded to its two bf16 terms (before instead of after the division by rms).
struct NormFold {
    const float *ss_in;     // consumer: per-block sums of squares of the producer, [32][SD_NORMFOLD_MAX_BLOCKS] (nullptr: operand is already normed)
    int32_t ss_nb;
    float eps;
    float *x;               // producer: residual rows [M][N], updated in place (nullptr: plain store)
    const float *g;         // producer: gains of the norm that follows, [N]
    float *ss_out;          // producer: [32][SD_NORMFOLD_MAX_BLOCKS], entry [m][block index]
    const int32_t *row_map; // operand row (and row of ss_in) of output row m (nullptr: m)
};
#define SD_NORMFOLD_MAX_BLOCKS 512

// Softmax partials the few-row GEMM can leave beside an LM head's logits, so that the draft sampler needs no pass
// over the whole row before it can place its uniform: for logits row m and block b (32 consecutive columns)
// p[(m * n_blocks + b) * 3 + {0, 1, 2}] = max, sum of exp((x - max) * invT) (0 when invT is 0: greedy), and the
// lowest column holding the max (an int stored bit for bit).
struct LmStats {
    float *p;   // nullptr: none wanted
    float invT; // 1 / temperature, or 0
};

// ---------------------------------------------------------------- host-side objects
struct sd_model {
    sd_model_config cfg;
    std::vector<const void *> wq, wk, wv, wo, wgate, wup, wdown;
    std::vector<const float *> norm_attn, norm_ffn;
    const void *embed, *lm_head;
    const float *final_norm;
    void *wmem;     // arena holding the model's own copy of every weight
    // low-rank adapters on q, k, v, o (fp32 on the device): a[p][layer] -> [n][rank][d], b[p][layer] -> [n][d][rank]
    int lora_n, lora_rank;
    float lora_scale;
    std::vector<const float *> lora_a[4], lora_b[4];
    void *lora_mem;
    int tiled_dd, tiled_fd, tiled_df, tiled_lm; // tile order used for [d][d], [F][d], [d][F], [V][d] matrices
    int esz; // bytes per weight / activation element
    int stream_nt; // 1: the weights (and with them the caches) of this model exceed the memory-side cache: stream them with the nontemporal hint
    // workspace (device)
    float *x;       // [max_rows][d] residual stream
    // activation buffers: fp32 models one plane, bf16 models two bf16 planes (hi, lo)
    void *abuf;     // [planes][max_rows][d] normed GEMM input
    float *qkv;     // [max_rows][3*d]
    void *qbuf;     // [planes][max_rows][d] rotated queries
    void *obuf;     // [planes][max_rows][d] attention output
    void *act;      // [planes][max_rows][d_ffn]
    size_t plane_d, plane_f; // element offsets between the planes
    float *logits;  // [max_rows][vocab]
    float *vstats;  // [max_rows][3] per-row (max, sum of exponentials, argmax) of the verify tail
    float *ss_part;  // [32][SD_NORMFOLD_MAX_BLOCKS] per-block sums of squares between a producer and its consumer (see NormFold)
    float *lm_stats; // [max_rows][vocab / 32][3] per-block softmax partials of the last LM head (see LmStats)
    int lm_stats_nb; // blocks per row the last forward's LM head left there (0: none)
    float *part;    // split-KV partial results of the attention kernel
    float *gpart_q, *gpart_r; // split-K partial slabs of the weight-streaming GEMMs (QKV; O / down)
    size_t gpart_q_floats, gpart_r_floats;
    size_t part_floats;
    float2 *rope;   // [max_pos][head_dim/2] (cos, sin)
    int32_t *plan_mem;
    PlanView plan;
    int last_lm_rows;
    int last_rows, last_a_rows; // rows of the last forward (layout of the step-major buffers); of abuf
};

struct sd_ctx {
    int B;
    int64_t total_cap;
    std::vector<int32_t> cap;
    std::vector<int64_t> off;
    int64_t *d_off;
    int32_t *d_cap, *d_tokens, *d_ntok, *d_kvlen, *d_status, *d_adapter;
    int32_t *d_gamma, *d_policy; // per-sequence candidate counts [B] (used when use_gamma) and accepted / examined [2][B]
    int use_gamma;
    int n_slots;
    sd_model *models[SD_MAX_SLOTS];
    void *kcache[SD_MAX_SLOTS];
    void *vcache[SD_MAX_SLOTS];
    int len_upper; // host upper bound of the longest sequence (tokens): sizes launches, never decides results
    int max_cap;   // largest sequence capacity (tokens)
    CtxView view() const
    {
        CtxView v;
        v.B = B;
        v.n_slots = n_slots;
        v.off = d_off;
        v.cap = d_cap;
        v.tokens = d_tokens;
        v.ntok = d_ntok;
        v.kvlen = d_kvlen;
        v.status = d_status;
        v.adapter = d_adapter;
        v.gam = use_gamma ? d_gamma : nullptr;
        v.pol = d_policy;
        return v;
    }
};

// ---------------------------------------------------------------- error plumbing
void sd_set_error(const std::string &s);
int sd_fail(int code, const std::string &s);
#define SD_HIP(expr)                                                                          \
    do {                                                                                      \
        hipError_t e__ = (expr);                                                              \
        if (e__ != hipSuccess)                                                                \
            return sd_fail(SD_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__));      \
    } while (0)

extern int g_force_generic;
extern int g_force_tile_cols;  // 96-row GEMM block width forced by option "gemm_tile_cols" (0 = automatic)
extern int g_rope_group;       // option "rope_group": RoPE + cache append one block per (head, row group) for bf16 models (1, default)
extern int g_prefill_attn;     // option "prefill_attn": the prefill attention kernel (1, default) or the split kernel per group (0)
extern int g_force_attn_waves; // fused attention block shape forced by option "attn_waves" (0 = automatic)
extern int g_stream_read_nt;   // sd_debug_stream_read: 1 = contiguous ranges with the nontemporal hint, 0 = grid-strided ordinary loads
extern int g_force_splits[3]; // per GEMM mode: K splits forced by option "gemm_splits" (0 = automatic)

// ---------------------------------------------------------------- kernel launchers
// (each returns a hipError_t from hipGetLastError after the launch)
// Low-rank update of n_proj (<= 3) projections that share the input rows X: for row r of a sequence with
// adapter a >= 0, out[r][p * N + n] (+)= scale * sum_j B[p][a][n][j] * (sum_k A[p][a][j][k] * X[r][k]); rows
// without an adapter (and projections whose factors are NULL) get 0 (or are left alone when accumulating).
hipError_t launch_lora_delta(hipStream_t s, int dtype, const void *X, ActView x_av, int M, int K, int N, int n_proj,
                             PlanView pv, const int32_t *adapter, int n_adapters, int rank, float scale,
                             const float *const *A, const float *const *B, float *out, int accumulate);
hipError_t launch_plan(hipStream_t s, int mode, int R, int n_seq, const int32_t *seq_ids, CtxView cv, int slot,
                       int upto_off, const int32_t *cand, int gamma, int cand_idx, int vocab, PlanView pv);
hipError_t launch_plan_prefill(hipStream_t s, int R, int G, int n_seq, const int32_t *seq_ids, CtxView cv, int slot,
                               int upto_off, int vocab, PlanView pv);
hipError_t launch_embed(hipStream_t s, int dtype, const void *E, const int32_t *row_tok, int M, int d, float *x);
hipError_t launch_embed_rmsnorm(hipStream_t s, int dtype, const void *E, const int32_t *row_tok, int M, int d, float *x,
                                const float *g, float eps, void *out, ActView out_av);
hipError_t launch_rmsnorm(hipStream_t s, int dtype, const float *x, const float *g, const int32_t *row_map,
                          int n_rows, int d, float eps, void *out, ActView out_av);
// row-major bf16 [N][K] -> tiled order (N % 16 == 0, K % 128 == 0); src and dst must not overlap
hipError_t launch_retile_bf16(hipStream_t s, const void *src, void *dst, int N, int K);
hipError_t launch_gemm_generic(hipStream_t s, int dtype, int mode, const void *A, ActView a_av, WeightSeg w, int M,
                               int N, int K, float *C, void *Cact, ActView c_av);
// (R: rows per plan slot; the rows of a slot hold consecutive positions of one sequence)
hipError_t launch_rope_append(hipStream_t s, int dtype, const float *qkv, int n_slabs, size_t slab_stride, PlanView pv,
                              CtxView cv, int M, int R, int H,
                              int hd, const float2 *rope, int max_pos, void *qbuf, ActView q_av, void *Kl, void *Vtl,
                              int64_t total_cap);
hipError_t launch_attn_generic(hipStream_t s, int dtype, const void *qbuf, ActView q_av, const void *Kl,
                               const void *Vtl, PlanView pv, CtxView cv, int R, int n_seq, int H, int hd,
                               int64_t total_cap, int len_upper, void *obuf, ActView o_av);
// stats / stats_nb: the per-block softmax partials the LM head left (LmStats), stats_nb blocks of 32 columns per
// row (0: none - the one-block-per-row samplers read the whole row first).  *did_embed: whether the sampler
// honoured next.embed (only the kernels that work from the partials do).
hipError_t launch_draft_sample(hipStream_t s, const float *logits, int n_seq, int V, float T, const float *u,
                               int gamma, int idx, int32_t *cand, float *q, const NextPlan &next,
                               const float *stats = nullptr, int stats_nb = 0, int *did_embed = nullptr);
hipError_t launch_verify_tail(hipStream_t s, const float *logits, int n_seq, int gamma, int V, float T,
                              const int32_t *cand, const float *q, const float *u, const int32_t *seq_ids,
                              int32_t *n_acc, int32_t *next_tok, int commit, CtxView cv, float *stats);
hipError_t launch_policy_choose(hipStream_t s, CtxView cv, const int32_t *seq_ids, int n_seq, double c_ratio, int gamma_max,
                                double alpha0, int32_t *gamma_all, int32_t *gammas_out);
hipError_t launch_commit(hipStream_t s, CtxView cv, const int32_t *seq_ids, int n_seq, int gamma,
                         const int32_t *cand, const int32_t *n_acc, const int32_t *next_tok);
hipError_t launch_route(hipStream_t s, const float *W, const float *b, int n_drafts, int emb, const float *e, int n,
                        int32_t *id);
hipError_t launch_set_kv(hipStream_t s, int dtype, const void *k_rows, const void *v_rows, int len, int H, int hd,
                         int64_t seq_off, int64_t total_cap, void *Kl, void *Vtl);

hipError_t launch_stream_read(hipStream_t s, const void *buf, size_t bytes, uint32_t *out);

// optimised bf16 paths (return hipErrorNotSupported when the shape is outside their domain)
// GEMM_STORE: C receives `splits` partial slabs (slab stride c_split_stride floats) that the consumer adds;
// GEMM_SWIGLU: Cact receives the bf16 hi/lo planes.  gemm_skinny_splits tells how many slabs to expect.
int gemm_skinny_splits(int mode, int M, int N, int K, int n_per_seg);
int gemm_normfold_blocks(int N);
int gemm_tile_plan(int mode, int M, int N, int K, int n_per_seg, int plan[6]); // host only: the row-blocked GEMM's launch plan // blocks of a NormFold producer launch with N output columns
// ls: softmax partials wanted beside the result (GEMM_STORE without K splits only); *ls_done tells whether the
// kernel chosen for the shape wrote them.
// nf: norm split between producer and consumer (few-row kernels only: the launcher returns
// hipErrorNotSupported for a shape it would send to the row-blocked kernel).
hipError_t launch_gemm_skinny_bf16(hipStream_t s, int mode, const void *A, ActView a_av, WeightSeg w, int M, int N,
                                   int K, float *C, size_t c_split_stride, int splits, void *Cact, ActView c_av,
                                   LmStats ls = {nullptr, 0.f}, int *ls_done = nullptr,
                                   NormFold nf = {nullptr, 0, 0.f, nullptr, nullptr, nullptr, nullptr});
hipError_t launch_add_rmsnorm(hipStream_t s, int dtype, float *x, const float *part, int n_slabs, size_t slab_stride,
                              const float *g, const int32_t *row_map, int n_rows, int d, float eps, void *out,
                              ActView out_av);
// wo_tiled / oslab (optional): let the attention blocks of a small model apply their head's columns of the
// output projection themselves and leave H partial slabs [H][n_seq * R][d_model] in oslab; *oproj_done tells
// whether they did (then obuf is not written and the projection launch is skipped).
#define SD_OPROJ_MAX_HEADS 16
hipError_t launch_attn_fused_bf16(hipStream_t s, const float *qkv, int n_slabs, size_t slab_stride, PlanView pv,
                                  CtxView cv, int R, int n_seq, int H, int hd, const float2 *rope, int max_pos,
                                  void *Kl, void *Vtl, int64_t total_cap, int len_upper, void *obuf, ActView o_av,
                                  int stream_nt, const void *wo_tiled = nullptr, int d_model = 0, float *oslab = nullptr,
                                  size_t oslab_floats = 0, int *oproj_done = nullptr);
hipError_t launch_attn_mfma_bf16(hipStream_t s, const void *qbuf, ActView q_av, const void *Kl, const void *Vtl,
                                 PlanView pv, CtxView cv, int R, int n_seq, int H, int hd, int64_t total_cap,
                                 int len_upper, float *part, size_t part_floats, void *obuf, ActView o_av, int stream_nt);
// Attention of a prefill forward: G > 1 groups of 16 rows per sequence (plan slots seq * G + g), rows already in the
// cache.  Returns hipErrorNotSupported outside its domain (the caller then takes the split kernel).
hipError_t launch_attn_prefill_bf16(hipStream_t s, const void *qbuf, ActView q_av, const void *Kl, const void *Vtl,
                                    PlanView pv, CtxView cv, int R, int n_seq, int G, int H, int hd, int64_t total_cap,
                                    int len_upper, float *part, size_t part_floats, void *obuf, ActView o_av);
