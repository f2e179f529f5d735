// bf16 multi-query-token decode attention on the matrix cores.
//
// For each (sequence, head) the R <= 16 new query rows (gamma+1 in verify, 1-2 in
// draft steps, up to 16 in prefill chunks) attend to the cached keys/values plus
// the rows appended in this forward, with a causal mask over the new positions:
// query row i sees cache rows [0, kv0 + i].  The work is streaming K and V once
// from HBM; the query rows ride along as one 16-wide MFMA operand, so the cost per
// cached token does not depend on gamma.
//
// Layout trick: scores are produced transposed, S^T[token][q] = K . Q^T, with the
// 16 rows of each K operand tile permuted (tile a: tokens 8*(i/4) + i%4, tile b:
// the same + 4).  The MFMA result then leaves every lane holding 8 consecutive
// tokens of one query row - exactly the operand layout of the second product
// O^T[d][q] = V^T[d][tokens] . P^T[tokens][q], whose V^T operand is a plain 16-byte
// load from the value cache, which is kept in transposed 32-token tiles ([head_dim][32],
// contiguous per tile).  No LDS, no shuffles between the two MFMAs.
// Queries arrive as two bf16 planes (hi + lo) and probabilities are split the same
// way, so both products carry ~16 mantissa bits of the activation operand; the
// softmax statistics stay in fp32.
//
// The KV range is split over blocks (flash-decoding style) and over the 4 waves
// of a block; partial (max, sum, O) triples are merged in LDS and, if there are
// several splits, by a small combine kernel.
//
// Paper (arXiv 2505.08600): Section 1, Figure 1b (parallel verification of the
// gamma candidates) and Figure 1a (draft steps).
#include "sd_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8; // explicit LDS address space: ds_read, not flat loads

#define AT_WAVES 4
#define AT_TILE 32
#define AT_NEG (-1.0e30f)

// Exponentials are the hardware 2^x (__builtin_amdgcn_exp2f): relative error of a few 1e-7 over the range softmax
// uses (arguments <= 0), far below the 2^-16 of the hi/lo split the probabilities go through next; -1e30 gives
// exactly 0.

union Pack8 {
    bf16x8 v;
    uint16_t u[8];
    uint32_t w[4];
};

// Scores of one 32-token tile -> probabilities (hi + lo operand of the second product) and the running softmax
// state of this lane's query row.  The scores arrive as S^T fragments: sa holds tokens tok0 + 0..3, sb tokens
// tok0 + 4..7 (tok0 = tile start + 8 * k-group).  sl2 = log2(e) / sqrt(head_dim): maxima and exponents are kept in
// the base-2 domain, p = 2^(s * sl2 - m), one multiply per score instead of two (every reader of m_run - the merges
// below and attn_combine_kernel - uses 2^x as well).  MASKED: tokens beyond `vis` are excluded; only tiles that
// reach into the new rows need it, and the others skip its compares and selects.  Returns the factor the
// accumulated output has to be scaled by (1 when the maximum stood).
// Maximum over the four 16-lane rows of a wave (lanes l, l ^ 16, l ^ 32, l ^ 48), left in every lane.  The two
// row-swap instructions of this part exchange rows between two registers inside the vector ALU; with both
// registers holding v, each lane ends up with its own value in one result and its partner's in the other.  (The
// general lane shuffle goes through the LDS unit: an address computation and a round trip per step.)
__device__ __forceinline__ float rows_max(float v)
{
    unsigned u = __float_as_uint(v);
    const auto r16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    v = fmaxf(__uint_as_float(r16[0]), __uint_as_float(r16[1]));
    u = __float_as_uint(v);
    const auto r32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r32[0]), __uint_as_float(r32[1]));
}

template <bool MASKED>
__device__ __forceinline__ float tile_softmax(const f32x4 &sa, const f32x4 &sb, float sl2, int tok0, int vis, float &m_run,
                                              float &l_run, Pack8 &ph, Pack8 &pl)
{
    float sc[8];
    float mx = AT_NEG;
#pragma unroll
    for (int e = 0; e < 8; e++) {
        float v = (e < 4 ? sa[e] : sb[e - 4]) * sl2;
        if (MASKED) v = tok0 + e <= vis ? v : AT_NEG;
        sc[e] = v;
        mx = fmaxf(mx, v);
    }
    mx = rows_max(mx);
    const float m_new = fmaxf(m_run, mx);
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new); // 1 when nothing changed, 0 from the initial state
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        float p0 = __builtin_amdgcn_exp2f(sc[e] - m_new), p1 = __builtin_amdgcn_exp2f(sc[e + 1] - m_new);
        if (MASKED) { // (a row that has seen nothing yet has m_new = AT_NEG: its differences are 0, not -inf)
            p0 = sc[e] > 0.5f * AT_NEG ? p0 : 0.f;
            p1 = sc[e + 1] > 0.5f * AT_NEG ? p1 : 0.f;
        }
        psum += p0;
        psum += p1;
        bf16x2_split(p0, p1, ph.w[e >> 1], pl.w[e >> 1]);
    }
    l_run = l_run * corr + psum;
    m_run = m_new;
    return corr;
}
// acc *= corr for the ND output tiles, as a branch the compiler keeps (it turns a plain `if` over these
// multiplies into selects that run for every tile, although the maxima settle after the first few)
#define SD_RESCALE_IF(cond, o, ND_, corr)                  \
    if (cond) {                                            \
        asm volatile("" ::: "memory");                     \
        _Pragma("unroll") for (int d_ = 0; d_ < ND_; d_++) { \
            o[d_][0] *= corr;                              \
            o[d_][1] *= corr;                              \
            o[d_][2] *= corr;                              \
            o[d_][3] *= corr;                              \
        }                                                  \
    }

// Online-softmax pass of one wave over the KV tiles t_begin, t_begin + t_stride, ... < t_end.
// qv/ql: hi and lo planes of the Q^T operand; vis: last visible token of this lane's query row.
// With Q_LDS the two planes are re-read from shared memory for every tile instead of living in
// registers (32 registers less, which is what lets an 8-wave block keep two tile buffers unspilled).
template <int HD, bool NT_HINT, bool Q_LDS = false>
__device__ __forceinline__ void attn_tiles(const uint16_t *__restrict__ K, const uint16_t *__restrict__ Vt,
                                           int64_t total_cap, const bf16x8 *qv, const bf16x8 *ql, int vis, int t_begin,
                                           int t_end, int t_stride, float &m_run, float &l_run, f32x4 *o)
{
    constexpr int NC = HD / 32;
    constexpr int ND = HD / 16;
    const int lane = threadIdx.x & 63;
    const int qi = lane & 15, grp = lane >> 4;
    const float sl2 = 1.44269504088896341f / sqrtf((float)HD);
    const int vis0 = __builtin_amdgcn_readfirstlane(vis); // (lane 0 holds row 0: the first new position; tiles that end before it need no mask)
    // K operand rows: lane row i holds token 8*(i/4) + i%4 (tile a) or that + 4 (tile b)
    // two register buffers: the loads of the next tile are in flight while the current one is consumed
    bf16x8 ka0[NC], kb0[NC], vv0[ND], ka1[NC], kb1[NC], vv1[ND];
    auto load_tile = [&](int t, bf16x8 *ka, bf16x8 *kb, bf16x8 *vv) {
        // MFMA c contracts head dimensions 32*c .. 32*c+31 (k-group grp takes 8 of them); the tile is stored
        // in operand order (kt_offset), so every load instruction reads one contiguous KiB
        const uint16_t *kp = K + (size_t)t * (AT_TILE * HD) + lane * 8;
#pragma unroll
        for (int c = 0; c < NC; c++) {
            ka[c] = ld_stream<NT_HINT>((const bf16x8 *)(kp + (2 * c) * 512));
            kb[c] = ld_stream<NT_HINT>((const bf16x8 *)(kp + (2 * c + 1) * 512));
        }
#pragma unroll
        for (int d = 0; d < ND; d++)
            vv[d] = ld_stream<NT_HINT>((const bf16x8 *)(Vt + (size_t)t * (AT_TILE * HD) + (d * 16 + qi) * AT_TILE + grp * 8));
    };
    auto compute_tile = [&](int t, const bf16x8 *ka, const bf16x8 *kb, const bf16x8 *vv) {
        const int t0 = t * AT_TILE;
        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NC; c++) {
            const bf16x8 qh = Q_LDS ? *(const volatile lds_bf16x8 *)(const lds_bf16x8 *)&qv[c * 4] : qv[c];
            const bf16x8 qo = Q_LDS ? *(const volatile lds_bf16x8 *)(const lds_bf16x8 *)&ql[c * 4] : ql[c];
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[c], qh, sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[c], qh, sb, 0, 0, 0);
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[c], qo, sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[c], qo, sb, 0, 0, 0);
        }
        // lane (q, grp) now holds scores of tokens t0 + 8*grp + e, e = 0..7 (sa: e<4, sb: e>=4)
        Pack8 ph, pl;
        const float corr = t0 + AT_TILE - 1 > vis0 ? tile_softmax<true>(sa, sb, sl2, t0 + 8 * grp, vis, m_run, l_run, ph, pl)
                                                   : tile_softmax<false>(sa, sb, sl2, t0 + 8 * grp, vis, m_run, l_run, ph, pl);
        // once the running maxima have settled corr is exactly 1 in every lane: skip the 4 * ND multiplies
        SD_RESCALE_IF(__any(corr != 1.0f), o, ND, corr)
#pragma unroll
        for (int d = 0; d < ND; d++) {
            o[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv[d], ph.v, o[d], 0, 0, 0);
            o[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv[d], pl.v, o[d], 0, 0, 0);
        }
    };
    int t = t_begin;
    if (t < t_end) load_tile(t, ka0, kb0, vv0);
    while (t < t_end) {
        const int tn = t + t_stride;
        if (tn < t_end) load_tile(tn, ka1, kb1, vv1);
        compute_tile(t, ka0, kb0, vv0);
        if (tn >= t_end) break;
        const int tnn = tn + t_stride;
        if (tnn < t_end) load_tile(tnn, ka0, kb0, vv0);
        compute_tile(tn, ka1, kb1, vv1);
        t = tnn;
    }
}

template <int HD, bool NT_HINT>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const uint16_t *__restrict__ qbuf, ActView q_av,
                                                        const uint16_t *__restrict__ Kl,
                                                        const uint16_t *__restrict__ Vtl, PlanView pv, CtxView cv,
                                                        int R, int H, int64_t total_cap, int S,
                                                        float *__restrict__ part, uint16_t *__restrict__ obuf,
                                                        ActView o_av)
{
    constexpr int NC = HD / 32; // 32-wide chunks of the head dimension (QK^T contraction)
    constexpr int ND = HD / 16; // 16-row tiles of V^T / O^T
    __shared__ float sO[AT_WAVES][ND][64][4];
    __shared__ float sM[AT_WAVES][16], sL[AT_WAVES][16];
    const int s = blockIdx.x, h = blockIdx.y;
    const int j = gridDim.z > 1 ? pv.seq_order[blockIdx.z] : 0; // longest sequences start first
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int qi = lane & 15, grp = lane >> 4;
    const int nq = pv.seq_nq[j], kv0 = pv.seq_kv0[j];
    const int Lk = kv0 + nq;
    const int64_t off = cv.off[pv.seq_b[j]];
    const int HDm = H * HD;
    const uint16_t *K = Kl + ((size_t)h * total_cap + off) * HD;
    const uint16_t *Vt = Vtl + ((size_t)h * total_cap + off) * HD; // this sequence's first 32-token tile
    // this block's tile range
    const int n_tiles = nq > 0 ? (Lk + AT_TILE - 1) / AT_TILE : 0; // nothing to do for unused sequences
    const int per = (n_tiles + S - 1) / S;
    const int t_begin = s * per, t_end = min(n_tiles, t_begin + per);
    // Q^T operand: lane (q, grp) holds Q[q][32*c + 8*grp .. +8], matching the K loads
    bf16x8 qv[NC], ql[NC];
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < NC; c++) {
        // 8 consecutive columns never straddle a 128-column step
        const bf16x8 *p = (const bf16x8 *)(qbuf + act_index(q_av, j * R + (qi < R ? qi : 0), h * HD + c * 32 + grp * 8, HDm));
        qv[c] = qi < nq ? *p : zero;
        ql[c] = qi < nq ? *(const bf16x8 *)((const uint16_t *)p + q_av.plane) : zero;
    }
    const int vis = kv0 + qi; // last visible token of this lane's query row
    float m_run = AT_NEG, l_run = 0.f;
    f32x4 o[ND];
#pragma unroll
    for (int d = 0; d < ND; d++) o[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
    attn_tiles<HD, NT_HINT>(K, Vt, total_cap, qv, ql, vis, t_begin + wave, t_end, AT_WAVES, m_run, l_run, o);
    // row sums were kept per k-group: finish them
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
#pragma unroll
    for (int d = 0; d < ND; d++)
#pragma unroll
        for (int r = 0; r < 4; r++) sO[wave][d][lane][r] = o[d][r];
    if (grp == 0) {
        sM[wave][qi] = m_run;
        sL[wave][qi] = l_run;
    }
    __syncthreads();
    // merge the 4 waves: element (d, slot, r) is O^T[dim = 16*d + 4*(slot/16) + r][q = slot%16]
    for (int e = threadIdx.x; e < ND * 256; e += 256) {
        const int d = e >> 8, slot = (e >> 2) & 63, r = e & 3;
        const int q = slot & 15, dim = 16 * d + 4 * (slot >> 4) + r;
        float M = AT_NEG;
#pragma unroll
        for (int w = 0; w < AT_WAVES; w++) M = fmaxf(M, sM[w][q]);
        float O = 0.f, L = 0.f;
#pragma unroll
        for (int w = 0; w < AT_WAVES; w++) {
            float f = __builtin_amdgcn_exp2f(sM[w][q] - M);
            O += sO[w][d][slot][r] * f;
            L += sL[w][q] * f;
        }
        if (q >= R) continue;
        if (S == 1) {
            float out = (q < nq && L > 0.f) ? O / L : 0.f;
            uint16_t hi = bf16_bits_rne(out);
            size_t oi = act_index(o_av, j * R + q, h * HD + dim, HDm);
            obuf[oi] = hi;
            obuf[oi + o_av.plane] = bf16_bits_rne(out - __uint_as_float((uint32_t)hi << 16));
        } else {
            float *pp = part + ((size_t)(j * H + h) * S + s) * 16 * (HD + 2);
            pp[q * HD + dim] = O;
            if (dim == 0) {
                pp[16 * HD + q] = M;
                pp[16 * HD + 16 + q] = L;
            }
        }
    }
}

// Merge the S split partials of each (sequence, head): one block per (head, sequence).
template <int HD, int SMAX = SD_ATTN_MAX_SPLITS>
__global__ void attn_combine_kernel(const float *__restrict__ part, PlanView pv, int R, int H, int S,
                                    uint16_t *__restrict__ obuf, ActView o_av)
{
    const int h = blockIdx.x, j = blockIdx.y;
    const int nq = pv.seq_nq[j];
    const float *base = part + (size_t)(j * H + h) * S * 16 * (HD + 2);
    for (int e = threadIdx.x; e < R * HD; e += blockDim.x) {
        const int q = e / HD, dim = e % HD;
        // all loads of the S (<= 32) partials are independent: issue them before the arithmetic
        float ms[SMAX], ls[SMAX], os[SMAX];
#pragma unroll
        for (int s = 0; s < SMAX; s++)
            if (s < S) {
                const float *pp = base + (size_t)s * 16 * (HD + 2);
                ms[s] = pp[16 * HD + q];
                ls[s] = pp[16 * HD + 16 + q];
                os[s] = pp[q * HD + dim];
            }
        float M = AT_NEG;
#pragma unroll
        for (int s = 0; s < SMAX; s++)
            if (s < S) M = fmaxf(M, ms[s]);
        float O = 0.f, L = 0.f;
#pragma unroll
        for (int s = 0; s < SMAX; s++)
            if (s < S) {
                float f = __builtin_amdgcn_exp2f(ms[s] - M);
                O += os[s] * f;
                L += ls[s] * f;
            }
        float out = (q < nq && L > 0.f) ? O / L : 0.f;
        uint16_t hi = bf16_bits_rne(out);
        size_t oi = act_index(o_av, j * R + q, h * HD + dim, H * HD);
        obuf[oi] = hi;
        obuf[oi + o_av.plane] = bf16_bits_rne(out - __uint_as_float((uint32_t)hi << 16));
    }
}

// Causal attention of a prompt (prefill): WG consecutive 16-row groups of ONE sequence and head per block, one
// group per wave.  With a block per group every group streams the whole prefix through L2 again (an 8192-token
// prompt at head width 128: 1.1 TB per 32 layers, the ceiling of what the L2s deliver); here the block stages
// each 32-token K / V tile in LDS once - double buffered, the loads of the next tile in flight while the
// current one is consumed - and every wave takes its operands from there, at the offsets it would have used in
// global memory (the tiles are stored in operand order, so the LDS reads are lane-linear), which divides the L2
// traffic by WG and leaves a wave ~100 registers, so that several blocks share a compute unit and cover each
// other's softmax and dependent MFMA chains.  The rows of all groups are in the cache before the launch
// (rope_append_kernel); wave w sees tokens <= kv0_w + row.  No merge between waves: each owns its rows.  With
// S > 1 the tile range is split over grid.z and attn_combine_kernel merges the partials (same layout as the
// split kernel's).  Blocks start with the longest prefixes first.
template <int HD, int WG>
__global__ __launch_bounds__(WG * 64, 3) void attn_prefill_kernel(const uint16_t *__restrict__ qbuf, ActView q_av,
                                                               const uint16_t *__restrict__ Kl,
                                                               const uint16_t *__restrict__ Vtl, PlanView pv, CtxView cv,
                                                               int R, int H, int G, int n_seq, int64_t total_cap, int S,
                                                               float *__restrict__ part, uint16_t *__restrict__ obuf,
                                                               ActView o_av)
{
    constexpr int NC = HD / 32, ND = HD / 16;
    constexpr int TILE = AT_TILE * HD;                   // elements of one K (or V) tile
    constexpr int NLD = (2 * TILE * 2) / (16 * WG * 64); // 16-byte pieces per thread and tile (K and V together)
    static_assert(NLD >= 1 && NLD * 16 * WG * 64 == 2 * TILE * 2, "tile does not divide over the block");
    __shared__ __attribute__((aligned(16))) uint16_t sKV[2][2 * TILE]; // [buffer][K tile, then V tile]
    const int h = blockIdx.x;
    const int n_gb = (G + WG - 1) / WG;
    const int seq = blockIdx.y % n_seq, gb = n_gb - 1 - blockIdx.y / n_seq; // later groups (longer prefixes) first
    const int s = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int qi = lane & 15, grp = lane >> 4;
    const int j0 = seq * G + gb * WG;
    const bool w_valid = gb * WG + wave < G;
    const int j = w_valid ? j0 + wave : j0;
    const int nq = w_valid ? pv.seq_nq[j] : 0, kv0 = pv.seq_kv0[j];
    // the block's tile range: up to the last row of its last non-empty group
    int lk_blk = 0;
#pragma unroll
    for (int w = 0; w < WG; w++)
        if (gb * WG + w < G) {
            const int nqw = pv.seq_nq[j0 + w];
            if (nqw > 0) lk_blk = max(lk_blk, pv.seq_kv0[j0 + w] + nqw);
        }
    const int n_tiles = (lk_blk + AT_TILE - 1) / AT_TILE;
    const int per = (n_tiles + S - 1) / S;
    const int t_begin = s * per, t_end = min(n_tiles, t_begin + per);
    const int64_t off = cv.off[pv.seq_b[j0]];
    const int HDm = H * HD;
    const uint16_t *K = Kl + ((size_t)h * total_cap + off) * HD;
    const uint16_t *Vt = Vtl + ((size_t)h * total_cap + off) * HD;
    // Q^T operand: lane (q, grp) holds Q[q][32*c + 8*grp .. +8]
    bf16x8 qv[NC], ql[NC];
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < NC; c++) {
        const bf16x8 *p = (const bf16x8 *)(qbuf + act_index(q_av, j * R + (qi < R ? qi : 0), h * HD + c * 32 + grp * 8, HDm));
        qv[c] = qi < nq ? *p : zero;
        ql[c] = qi < nq ? *(const bf16x8 *)((const uint16_t *)p + q_av.plane) : zero;
    }
    const int vis = kv0 + qi;             // last visible token of this lane's query row
    const int vis_wave = nq > 0 ? kv0 + nq - 1 : -1; // ... of the wave's last row
    const float sl2 = 1.44269504088896341f / sqrtf((float)HD);
    float m_run = AT_NEG, l_run = 0.f;
    f32x4 o[ND];
#pragma unroll
    for (int d = 0; d < ND; d++) o[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // staging: piece c = threadIdx.x + k * threads of the tile pair; pieces 0 .. TILE/8-1 are K, the rest V.  Two
    // register sets: the loads of tiles t + 1 and t + 2 are in flight while tile t is consumed (one tile ahead left
    // every iteration waiting for most of a memory round trip)
    bf16x8 st0[NLD], st1[NLD];
    // The K tile is stored in operand order already: piece c goes to LDS position c and a fragment read is
    // lane-linear.  The V^T tile is [dim][32 tokens] (64-byte rows), and lane (qi, grp) of a fragment read wants piece
    // grp of row 16 d + qi: read from a row-major copy, such reads hit the banks unevenly (80 % of the LDS cycles were
    // conflict cycles).  So the thread that fills LDS position 64 d + l of the V part fetches the piece lane l of
    // fragment d will want - row 16 d + l % 16, piece l / 16.  The lanes of a wave still cover the same contiguous
    // KiB of global memory, only in another order, and both the LDS writes and the fragment reads are linear.
    auto fetch = [&](int t, bf16x8 *st) {
#pragma unroll
        for (int k = 0; k < NLD; k++) {
            const int c = threadIdx.x + k * (WG * 64);
            const int cv = c - TILE / 8, l = cv & 63;
            const uint16_t *src = c < TILE / 8 ? K + (size_t)t * TILE + c * 8
                                               : Vt + (size_t)t * TILE + ((((cv >> 6) * 16 + (l & 15)) << 2) + (l >> 4)) * 8;
            st[k] = *(const bf16x8 *)src;
        }
    };
    auto stash = [&](int b, const bf16x8 *st) {
#pragma unroll
        for (int k = 0; k < NLD; k++) *(lds_bf16x8 *)(lds_bf16x8 *)&sKV[b][(threadIdx.x + k * (WG * 64)) * 8] = st[k];
    };
    auto consume = [&](int t, int b) {
    if (t * AT_TILE <= vis_wave) { // (uniform over the wave) tiles past the wave's last row hold nothing it sees
        const uint16_t *kp = &sKV[b][lane * 8];
        const uint16_t *vp = &sKV[b][TILE + lane * 8]; // (fragment d: + 512 d elements)
        // all K fragments are requested before the first product, and half of the V fragments behind the score
        // products (into the registers the K fragments leave), so that the LDS round trips run under the MFMAs and
        // the softmax instead of in front of every pair of products
        bf16x8 kf[2 * NC];
#pragma unroll
        for (int c = 0; c < 2 * NC; c++) kf[c] = *(const lds_bf16x8 *)(const lds_bf16x8 *)(kp + c * 512);
        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NC; c++) {
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[2 * c], qv[c], sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[2 * c + 1], qv[c], sb, 0, 0, 0);
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[2 * c], ql[c], sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[2 * c + 1], ql[c], sb, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        constexpr int NVH = ND / 2; // (all of them would not fit three waves per SIMD without spilling)
        bf16x8 vf[NVH];
#pragma unroll
        for (int d = 0; d < NVH; d++) vf[d] = *(const lds_bf16x8 *)(const lds_bf16x8 *)(vp + d * 512);
        __builtin_amdgcn_sched_barrier(0);
        // lane (q, grp) holds the scores of tokens 32 t + 8 grp + e, e = 0..7 (sa: e < 4, sb: e >= 4)
        const int t0 = t * AT_TILE;
        Pack8 ph, pl;
        const float corr = t0 + AT_TILE - 1 > kv0 ? tile_softmax<true>(sa, sb, sl2, t0 + 8 * grp, vis, m_run, l_run, ph, pl)
                                                  : tile_softmax<false>(sa, sb, sl2, t0 + 8 * grp, vis, m_run, l_run, ph, pl);
        SD_RESCALE_IF(__any(corr != 1.0f), o, ND, corr)
#pragma unroll
        for (int d = 0; d < ND; d++) {
            const bf16x8 vv = d < NVH ? vf[d] : *(const lds_bf16x8 *)(const lds_bf16x8 *)(vp + d * 512);
            o[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv, ph.v, o[d], 0, 0, 0);
            o[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv, pl.v, o[d], 0, 0, 0);
        }
    }
    };
    // one step: tile t sits in LDS buffer b; `nxt` holds tile t + 1 (requested earlier), `far` is free for tile t + 2
    auto step = [&](int t, int b, bf16x8 *nxt, bf16x8 *far) {
        fetch(min(t + 2, t_end - 1), far); // (always issued, so that the wait for `nxt` below counts exactly)
        consume(t, b);
        if (t + 1 < t_end) stash(b ^ 1, nxt);
        __syncthreads(); // tile t + 1 is staged, and nobody reads buffer b any more
    };
    if (t_begin < t_end) {
        fetch(t_begin, st0);
        if (t_begin + 1 < t_end) fetch(t_begin + 1, st1);
        stash(0, st0);
    }
    __syncthreads();
    for (int t = t_begin; t < t_end; t += 2) {
        step(t, 0, st1, st0);
        if (t + 1 < t_end) step(t + 1, 1, st0, st1);
    }
    if (!w_valid) return;
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    // lane (q = qi, grp) holds O^T[dim = 16 d + 4 grp + r][q] in o[d][r]
    if (qi >= R) return;
    if (S == 1) {
        const bool live = qi < nq && l_run > 0.f;
#pragma unroll
        for (int d = 0; d < ND; d++) {
            float out[4];
#pragma unroll
            for (int r = 0; r < 4; r++) out[r] = live ? o[d][r] / l_run : 0.f;
            uint32_t h0, l0, h1, l1;
            bf16x2_split(out[0], out[1], h0, l0);
            bf16x2_split(out[2], out[3], h1, l1);
            const size_t oi = act_index(o_av, j * R + qi, h * HD + 16 * d + 4 * grp, HDm); // 4 columns inside one K step
            *(uint2 *)(obuf + oi) = make_uint2(h0, h1);
            *(uint2 *)(obuf + oi + o_av.plane) = make_uint2(l0, l1);
        }
    } else {
        float *pp = part + ((size_t)(j * H + h) * S + s) * 16 * (HD + 2);
#pragma unroll
        for (int d = 0; d < ND; d++) *(f32x4 *)(pp + qi * HD + 16 * d + 4 * grp) = o[d];
        if (grp == 0) {
            pp[16 * HD + qi] = m_run;
            pp[16 * HD + 16 + qi] = l_run;
        }
    }
}

// Fused RoPE + cache append + attention for one (sequence, head) per block, no KV split: used when
// there are enough (sequence, head) pairs to fill the chip or the context is short, where the split
// kernel plus its combine pass and the separate RoPE kernel are three latency-bound launches.
// The block first adds the split-K slabs of the QKV GEMM for its head, rotates q and k, writes the new
// K / V rows into the cache in place and q (hi, lo) into LDS; after a barrier its waves stream the cache
// (including the rows just written) tile by tile, and merge their partial results in LDS.
// WAVES = 8: one block per compute unit (few blocks, each as parallel as possible); WAVES = 4: two
// resident blocks per unit, so one block's prologue and merge overlap the other's streaming (many blocks).
// OPROJ (small models, few blocks): the block goes on to multiply its head's output rows with the head's
// HD columns of the output projection - Wo[:, h * HD .. + HD], tiled order - and stores the [R][d_model] partial
// sums as slab h of `oslab`; the add + norm kernel that follows adds the H slabs to the residual.  The separate
// projection launch and the round trip of the attention output through memory disappear, which is what such a
// forward spends its time on; a head's slice of Wo is d_model * HD * 2 bytes (98 KB for 768 x 64).  The output
// rows are split into hi + lo exactly as they are when stored for the GEMM.
struct OProj {
    const uint16_t *Wo; // tiled [d_model][d_model]
    float *oslab;       // [H][rows][d_model]
    size_t slab_stride; // rows * d_model
    int32_t d_model;
};
template <int HD, int WAVES, bool NT_HINT, bool OPROJ>
__global__ __launch_bounds__(WAVES * 64, 2) void attn_fused_kernel(const float *__restrict__ qkv, int n_slabs,
                                                                   size_t slab_stride, PlanView pv, CtxView cv, int R,
                                                                   int H, const float2 *__restrict__ rope, int max_pos,
                                                                   uint16_t *__restrict__ Kl, uint16_t *__restrict__ Vtl,
                                                                   int64_t total_cap, uint16_t *__restrict__ obuf,
                                                                   ActView o_av, OProj op)
{
    constexpr int ND = HD / 16;
    constexpr int HALF = HD / 2;
    __shared__ float sO[WAVES][ND][64][4];
    __shared__ float sM[WAVES][16], sL[WAVES][16];
    __shared__ __attribute__((aligned(16))) uint16_t sQ[2][16][HD];
    const int h = blockIdx.x;
    const int j = gridDim.y > 1 ? pv.seq_order[blockIdx.y] : 0; // longest sequences start first
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int qi = lane & 15, grp = lane >> 4;
    const int nq = pv.seq_nq[j], kv0 = pv.seq_kv0[j];
    const int Lk = kv0 + nq;
    const int64_t off = cv.off[pv.seq_b[j]];
    const int HDm = H * HD;
    uint16_t *K = Kl + ((size_t)h * total_cap + off) * HD;
    uint16_t *Vt = Vtl + ((size_t)h * total_cap + off) * HD; // this sequence's first 32-token tile
    // ---- prologue: slabs -> q, k, v of this head; RoPE; append
    {
        for (int idx = threadIdx.x; idx < 16 * HALF; idx += WAVES * 64) {
            const int r = idx / HALF, e = idx % HALF;
            const int row = j * R + (r < R ? r : 0);
            const int pos = kv0 + r;
            bool valid = r < nq && pos < max_pos;
            if (r < nq && pos >= max_pos && e == 0) atomicOr(cv.status, 8);
            float q0 = 0.f, q1 = 0.f, k0 = 0.f, k1 = 0.f, v0 = 0.f, v1 = 0.f;
            if (valid) {
                const float *base = qkv + (size_t)row * 3 * HDm + h * HD + e;
                float ld[8][6];
#pragma unroll
                for (int sl = 0; sl < 8; sl++)
                    if (sl < n_slabs) {
                        const float *rs = base + (size_t)sl * slab_stride;
                        ld[sl][0] = rs[0];
                        ld[sl][1] = rs[HALF];
                        ld[sl][2] = rs[HDm];
                        ld[sl][3] = rs[HDm + HALF];
                        ld[sl][4] = rs[2 * HDm];
                        ld[sl][5] = rs[2 * HDm + HALF];
                    }
#pragma unroll
                for (int sl = 0; sl < 8; sl++)
                    if (sl < n_slabs) {
                        q0 += ld[sl][0];
                        q1 += ld[sl][1];
                        k0 += ld[sl][2];
                        k1 += ld[sl][3];
                        v0 += ld[sl][4];
                        v1 += ld[sl][5];
                    }
                const float2 cs = rope[(size_t)pos * HALF + e];
                const float qa = q0 * cs.x - q1 * cs.y, qb = q1 * cs.x + q0 * cs.y;
                const float ka = k0 * cs.x - k1 * cs.y, kb = k1 * cs.x + k0 * cs.y;
                q0 = qa;
                q1 = qb;
                K[kt_offset(HD, pos, e)] = bf16_bits_rne(ka);
                K[kt_offset(HD, pos, e + HALF)] = bf16_bits_rne(kb);
                Vt[vt_offset(HD, pos, e)] = bf16_bits_rne(v0);
                Vt[vt_offset(HD, pos, e + HALF)] = bf16_bits_rne(v1);
            }
            const uint16_t h0 = bf16_bits_rne(q0), h1 = bf16_bits_rne(q1);
            sQ[0][r][e] = h0;
            sQ[0][r][e + HALF] = h1;
            sQ[1][r][e] = bf16_bits_rne(q0 - __uint_as_float((uint32_t)h0 << 16));
            sQ[1][r][e + HALF] = bf16_bits_rne(q1 - __uint_as_float((uint32_t)h1 << 16));
        }
    }
    __syncthreads(); // q in LDS; the new cache rows are visible to this block's later loads
    // the Q^T operand stays in LDS: lane (q, grp) reads Q[q][32*c + 8*grp .. +8] per tile
    const bf16x8 *qv = (const bf16x8 *)(&sQ[0][qi][grp * 8]);
    const bf16x8 *ql = (const bf16x8 *)(&sQ[1][qi][grp * 8]);
    const int n_tiles = nq > 0 ? (Lk + AT_TILE - 1) / AT_TILE : 0;
    const int vis = kv0 + qi;
    float m_run = AT_NEG, l_run = 0.f;
    f32x4 o[ND];
#pragma unroll
    for (int d = 0; d < ND; d++) o[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
    attn_tiles<HD, NT_HINT, true>(K, Vt, total_cap, qv, ql, vis, wave, n_tiles, WAVES, m_run, l_run, o);
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    // OPROJ: this wave's 16-column tiles of the projection are wave, wave + WAVES, ...; their weight fragments
    // (operand order: one contiguous KiB per instruction) are requested now and arrive during the merge
    constexpr int OPF = OPROJ ? (HD == 64 ? 8 : 4) : 1, OKI = HD / 32;
    bf16x8 wf[OPF][OKI];
    if (OPROJ) {
        const int n_ot = op.d_model >> 4;
#pragma unroll
        for (int t = 0; t < OPF; t++) {
            const int nt = wave + t * WAVES;
#pragma unroll
            for (int i = 0; i < OKI; i++) {
                const int kabs = h * HD + 32 * i;
                const uint16_t *wp = op.Wo + ((size_t)(nt < n_ot ? nt : 0) * (op.d_model >> 7) + (kabs >> 7)) * 2048 +
                                     ((kabs & 127) >> 5) * 512 + lane * 8;
                wf[t][i] = *(const bf16x8 *)wp;
            }
        }
    }
    // ---- merge: every wave leaves its (max, sum, O) in LDS; after one barrier the block combines them
#pragma unroll
    for (int d = 0; d < ND; d++)
#pragma unroll
        for (int r = 0; r < 4; r++) sO[wave][d][lane][r] = o[d][r];
    if (grp == 0) {
        sM[wave][qi] = m_run;
        sL[wave][qi] = l_run;
    }
    __syncthreads();
    // one thread per (d tile, lane slot): four consecutive head dimensions of one query row
    for (int e = threadIdx.x; e < ND * 64; e += WAVES * 64) {
        const int d = e >> 6, slot = e & 63;
        const int q = slot & 15, dim = 16 * d + 4 * (slot >> 4);
        if (q >= R) continue;
        float M = AT_NEG;
#pragma unroll
        for (int w = 0; w < WAVES; w++) M = fmaxf(M, sM[w][q]);
        f32x4 O = {0.f, 0.f, 0.f, 0.f};
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; w++) {
            const float f = __builtin_amdgcn_exp2f(sM[w][q] - M);
            const f32x4 p = *(const f32x4 *)&sO[w][d][slot][0];
            O += p * f;
            L += sL[w][q] * f;
        }
        const bool live = q < nq && L > 0.f;
        float out[4];
#pragma unroll
        for (int r = 0; r < 4; r++) out[r] = live ? O[r] / L : 0.f;
        uint32_t h0, l0, h1, l1;
        bf16x2_split(out[0], out[1], h0, l0);
        bf16x2_split(out[2], out[3], h1, l1);
        if (OPROJ) { // (q no longer needed: its LDS rows take the output rows, same [plane][row][dim] layout)
            *(uint2 *)&sQ[0][q][dim] = make_uint2(h0, h1);
            *(uint2 *)&sQ[1][q][dim] = make_uint2(l0, l1);
        } else {
            const size_t oi = act_index(o_av, j * R + q, h * HD + dim, HDm); // 4 columns inside one K step
            *(uint2 *)(obuf + oi) = make_uint2(h0, h1);
            *(uint2 *)(obuf + oi + o_av.plane) = make_uint2(l0, l1);
        }
    }
    if (OPROJ) {
        __syncthreads();
        // D[n][m] = sum_k Wo[n][h * HD + k] * out[m][k]: weights as the first operand, lane (m = qi, grp) of the
        // second holds out[m][32 i + 8 grp .. + 8]; the result leaves n = 4 grp + r, m = qi in acc[r]
        const int n_ot = op.d_model >> 4;
        float *dst = op.oslab + (size_t)h * op.slab_stride + (size_t)(j * R + qi) * op.d_model + 4 * grp;
#pragma unroll
        for (int t = 0; t < OPF; t++) {
            const int nt = wave + t * WAVES;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < OKI; i++) {
                const bf16x8 ah = *(const lds_bf16x8 *)&sQ[0][qi][32 * i + grp * 8];
                const bf16x8 al = *(const lds_bf16x8 *)&sQ[1][qi][32 * i + grp * 8];
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[t][i], ah, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[t][i], al, acc, 0, 0, 0);
            }
            if (nt < n_ot && qi < R) *(f32x4 *)(dst + nt * 16) = acc;
        }
    }
}

int g_force_attn_waves = 0;

// Returns hipErrorNotSupported when the split path (RoPE kernel + split attention + combine) should run.
hipError_t launch_attn_fused_bf16(hipStream_t s, const float *qkv, int n_slabs, size_t slab_stride, PlanView pv,
                                  CtxView cv, int R, int n_seq, int H, int hd, const float2 *rope, int max_pos,
                                  void *Kl, void *Vtl, int64_t total_cap, int len_upper, void *obuf, ActView o_av,
                                  int stream_nt, const void *wo_tiled, int d_model, float *oslab, size_t oslab_floats,
                                  int *oproj_done)
{
    if (oproj_done) *oproj_done = 0;
    if (R < 1 || R > 16 || (hd != 64 && hd != 128) || n_slabs < 1 || n_slabs > 8) return hipErrorNotSupported;
    if (n_seq > 65535 || H > 65535) return hipErrorNotSupported;
    const int tiles_upper = (len_upper + AT_TILE - 1) / AT_TILE;
    // one block per (sequence, head): fine when every wave has at most a few tiles anyway, or when those blocks
    // alone fill the chip and the contexts stay below about 2000 tokens - beyond that the split kernel, whose blocks
    // only stream, is faster even with its RoPE and combine launches (32 x 2048 tokens, 40 heads: 20.1 against
    // 20.4 ms for the whole verify pass; 64 sequences of 1024 - 8192 tokens: 38.0 against 38.6; at 32 sequences of
    // up to 1024 tokens the fused kernel wins, 8.26 against 8.50 ms)
    if (!(tiles_upper <= 48 || ((long)n_seq * H >= 512 && tiles_upper < 64))) return hipErrorNotSupported;
    // with more than two blocks per compute unit and short contexts the 4-wave shape (two resident blocks
    // per unit) hides each block's prologue and merge behind its neighbour's streaming; from about 40 tiles
    // per block on, the 8-wave shape streams faster (measured: 4.9 against 4.6 TB/s at 2048 tokens, 5.5
    // against 5.2 at 1024..8192)
    const bool many = g_force_attn_waves ? g_force_attn_waves == 4 : ((long)n_seq * H >= 512 && tiles_upper <= 40);
    dim3 grid(H, n_seq), block(many ? 256 : 512);
    // output projection inside the block: small models in few blocks (each block reads its head's slice of Wo;
    // 8 waves x 8 (head width 64) or 4 (128) column tiles bound d_model), H slabs for the add + norm kernel
    const size_t rows = (size_t)n_seq * R;
    const bool oproj = wo_tiled && oslab && !many && stream_nt == 0 && d_model % 128 == 0 && d_model == H * hd &&
                       d_model <= 16 * 8 * (hd == 64 ? 8 : 4) && H <= SD_OPROJ_MAX_HEADS && (long)n_seq * H < 512 &&
                       (size_t)H * rows * d_model <= oslab_floats && ((uintptr_t)wo_tiled & 15) == 0;
    const OProj op = {(const uint16_t *)wo_tiled, oslab, rows * (size_t)d_model, d_model};
    if (oproj) {
        if (hd == 128)
            hipLaunchKernelGGL((attn_fused_kernel<128, 8, false, true>), grid, block, 0, s, qkv, n_slabs, slab_stride, pv, cv,
                               R, H, rope, max_pos, (uint16_t *)Kl, (uint16_t *)Vtl, total_cap, (uint16_t *)obuf, o_av, op);
        else
            hipLaunchKernelGGL((attn_fused_kernel<64, 8, false, true>), grid, block, 0, s, qkv, n_slabs, slab_stride, pv, cv,
                               R, H, rope, max_pos, (uint16_t *)Kl, (uint16_t *)Vtl, total_cap, (uint16_t *)obuf, o_av, op);
        if (oproj_done) *oproj_done = 1;
        return hipGetLastError();
    }
#define SD_FUSED(HD_, WAVES_)                                                                                          \
    do {                                                                                                               \
        if (stream_nt)                                                                                                 \
            hipLaunchKernelGGL((attn_fused_kernel<HD_, WAVES_, true, false>), grid, block, 0, s, qkv, n_slabs,         \
                               slab_stride, pv, cv, R, H, rope, max_pos, (uint16_t *)Kl, (uint16_t *)Vtl, total_cap,   \
                               (uint16_t *)obuf, o_av, op);                                                            \
        else                                                                                                           \
            hipLaunchKernelGGL((attn_fused_kernel<HD_, WAVES_, false, false>), grid, block, 0, s, qkv, n_slabs,        \
                               slab_stride, pv, cv, R, H, rope, max_pos, (uint16_t *)Kl, (uint16_t *)Vtl, total_cap,   \
                               (uint16_t *)obuf, o_av, op);                                                            \
    } while (0)
    if (hd == 128) {
        if (many) SD_FUSED(128, 4);
        else SD_FUSED(128, 8);
    } else {
        if (many) SD_FUSED(64, 4);
        else SD_FUSED(64, 8);
    }
#undef SD_FUSED
    return hipGetLastError();
}

hipError_t launch_attn_mfma_bf16(hipStream_t s, const void *qbuf, ActView q_av, const void *Kl, const void *Vtl,
                                 PlanView pv, CtxView cv, int R, int n_seq, int H, int hd, int64_t total_cap,
                                 int len_upper, float *part, size_t part_floats, void *obuf, ActView o_av, int stream_nt)
{
    if (R < 1 || R > 16 || (hd != 64 && hd != 128)) return hipErrorNotSupported;
    if (n_seq > 65535 || H > 65535) return hipErrorNotSupported;
    int tiles_upper = (len_upper + AT_TILE - 1) / AT_TILE;
    int S = (tiles_upper + AT_WAVES - 1) / AT_WAVES;                  // at least one tile per wave
    int want = (512 + n_seq * H - 1) / (n_seq * H);                   // enough blocks to fill the chip
    if (S > want) S = want;
    if (S > SD_ATTN_MAX_SPLITS) S = SD_ATTN_MAX_SPLITS;
    while (S > 1 && (size_t)n_seq * H * S * 16 * (hd + 2) > part_floats) S--;
    if (S < 1) S = 1;
    dim3 grid(S, H, n_seq), block(256);
#define SD_SPLIT_ATTN(HD_, NT_)                                                                                      \
    hipLaunchKernelGGL((attn_mfma_kernel<HD_, NT_>), grid, block, 0, s, (const uint16_t *)qbuf, q_av,                \
                       (const uint16_t *)Kl, (const uint16_t *)Vtl, pv, cv, R, H, total_cap, S, part, (uint16_t *)obuf, \
                       o_av)
    if (hd == 128) {
        if (stream_nt) SD_SPLIT_ATTN(128, true);
        else SD_SPLIT_ATTN(128, false);
    } else {
        if (stream_nt) SD_SPLIT_ATTN(64, true);
        else SD_SPLIT_ATTN(64, false);
    }
#undef SD_SPLIT_ATTN
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || S == 1) return e;
    if (hd == 128)
        hipLaunchKernelGGL(attn_combine_kernel<128>, dim3(H, n_seq), dim3(256), 0, s, part, pv, R, H, S,
                           (uint16_t *)obuf, o_av);
    else
        hipLaunchKernelGGL(attn_combine_kernel<64>, dim3(H, n_seq), dim3(256), 0, s, part, pv, R, H, S,
                           (uint16_t *)obuf, o_av);
    return hipGetLastError();
}

int g_prefill_attn = 1; // option "prefill_attn": 0 sends prefill forwards through the split kernel, one block set per group

// Attention of a prefill forward (G > 1 groups of 16 rows per sequence; all rows already in the cache).
hipError_t launch_attn_prefill_bf16(hipStream_t s, const void *qbuf, ActView q_av, const void *Kl, const void *Vtl,
                                    PlanView pv, CtxView cv, int R, int n_seq, int G, int H, int hd, int64_t total_cap,
                                    int len_upper, float *part, size_t part_floats, void *obuf, ActView o_av)
{
    if (!g_prefill_attn || R != 16 || G < 2 || (hd != 64 && hd != 128)) return hipErrorNotSupported;
    constexpr int WG = 4;
    const int n_gb = (G + WG - 1) / WG, n_slots = n_seq * G;
    if ((long)n_seq * n_gb > 65535 || H > 65535) return hipErrorNotSupported;
    const int tiles_upper = (len_upper + AT_TILE - 1) / AT_TILE;
    // as many splits as keep all blocks resident at once (three per compute unit at head width 128), at least 8
    // tiles per split, and partials that fit
    int S = 768 / (H * n_seq * n_gb);
    if (S > tiles_upper / 8) S = tiles_upper / 8;
    if (S > SD_ATTN_MAX_SPLITS) S = SD_ATTN_MAX_SPLITS;
    while (S > 1 && (size_t)n_slots * H * S * 16 * (hd + 2) > part_floats) S--;
    if (S < 1) S = 1;
    dim3 grid(H, n_seq * n_gb, S), block(WG * 64);
    if (hd == 128)
        hipLaunchKernelGGL((attn_prefill_kernel<128, WG>), grid, block, 0, s, (const uint16_t *)qbuf, q_av,
                           (const uint16_t *)Kl, (const uint16_t *)Vtl, pv, cv, R, H, G, n_seq, total_cap, S, part,
                           (uint16_t *)obuf, o_av);
    else
        hipLaunchKernelGGL((attn_prefill_kernel<64, WG>), grid, block, 0, s, (const uint16_t *)qbuf, q_av,
                           (const uint16_t *)Kl, (const uint16_t *)Vtl, pv, cv, R, H, G, n_seq, total_cap, S, part,
                           (uint16_t *)obuf, o_av);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || S == 1) return e;
    // (the unrolled loops of the combine kernel cover its template's split count: short ones for the usual 2 - 8)
    if (hd == 128 && S <= 4)
        hipLaunchKernelGGL((attn_combine_kernel<128, 4>), dim3(H, n_slots), dim3(256), 0, s, part, pv, R, H, S, (uint16_t *)obuf,
                           o_av);
    else if (hd == 128 && S <= 8)
        hipLaunchKernelGGL((attn_combine_kernel<128, 8>), dim3(H, n_slots), dim3(256), 0, s, part, pv, R, H, S, (uint16_t *)obuf,
                           o_av);
    else if (hd == 128)
        hipLaunchKernelGGL((attn_combine_kernel<128>), dim3(H, n_slots), dim3(256), 0, s, part, pv, R, H, S, (uint16_t *)obuf,
                           o_av);
    else if (S <= 4)
        hipLaunchKernelGGL((attn_combine_kernel<64, 4>), dim3(H, n_slots), dim3(256), 0, s, part, pv, R, H, S, (uint16_t *)obuf,
                           o_av);
    else if (S <= 8)
        hipLaunchKernelGGL((attn_combine_kernel<64, 8>), dim3(H, n_slots), dim3(256), 0, s, part, pv, R, H, S, (uint16_t *)obuf,
                           o_av);
    else
        hipLaunchKernelGGL((attn_combine_kernel<64>), dim3(H, n_slots), dim3(256), 0, s, part, pv, R, H, S, (uint16_t *)obuf,
                           o_av);
    return hipGetLastError();
}
