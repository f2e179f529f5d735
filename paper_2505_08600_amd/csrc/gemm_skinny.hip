// bf16 weight-streaming GEMMs: C[M][N] = A[M][K] . W[N][K]^T for the decoder's linear layers.
//
// At batch 1 (M = gamma+1 verify rows, or one draft row) the work is reading each
// weight once from HBM, so the kernels are organised around the weight stream and
// the matrix cores only keep the ALUs out of the way; at batch 32-64 (M = 192-576)
// the same weight stream feeds enough rows for the matrix cores to matter.
//
//  * weights are stored in 16-row x 128-element tiles in MFMA operand order, so each
//    of the four load instructions of a K step reads one contiguous kilobyte straight
//    into operand registers (v_mfma_f32_16x16x32_bf16: lane l supplies row l%16,
//    k-group l/16).  Row-major weights would spread every such load over 16 rows 2K
//    bytes apart, which lands on one L2 channel and limits a compute unit to about a
//    third of the rate it reaches on the tiles;
//  * activations are two bf16 planes (hi + lo, ~16 mantissa bits).  For M <= 8 both
//    planes ride in ONE operand: MFMA columns 0..7 carry the hi rows, columns 8..15
//    the lo rows, and the epilogue adds the two halves; for larger M every weight
//    fragment is multiplied twice;
//  * M <= 32 (gemm_ksplit_kernel): the waves of a block split K, fetch their
//    activation fragments straight from L2 and meet in LDS - no barrier in the K loop;
//    M > 32 (gemm_tile_kernel): 48-row blocks share a staged activation chunk in LDS;
//  * results leave either directly (store; SwiGLU: silu(gate)*up split to bf16
//    hi/lo) or as fp32 partial sums per K split, which the consuming kernel adds in
//    a fixed order (the fused attention prologue for QKV, add_rmsnorm for the residual
//    GEMMs), so results are bit-reproducible run to run.
//
// Paper (arXiv 2505.08600): Section 1, Figure 1 (draft steps and the parallel
// verify pass whose linear layers these are); Section 3.1 (LLaMA blocks).
#include "sd_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Pins the program order of the memory operations around it, for the optimiser and the scheduler alike.
#define SD_ORDER()                          \
    do {                                    \
        asm volatile("" ::: "memory");       \
        __builtin_amdgcn_sched_barrier(0);  \
    } while (0)
#define GS_PAD 8 // row padding in LDS (16 bytes): operand rows fall into distinct banks

// Row-blocked GEMM for M > 32 (batched verify, prefill chunks of many sequences).
// MODE: GEMM_STORE (C = acc, or partial sums when grid.y > 1) / GEMM_SWIGLU (the block's WAVES * NT tiles are,
// alternately, the gate and the up tile of WAVES * NT / 2 groups of 16 output columns; tile q belongs to wave
// q / NT, so with an odd NT every second pair straddles two waves and the gate accumulators change wave
// through LDS before the epilogue; a last block may hold fewer pairs than the others).  A block owns BM rows (hi plane in operand rows 0..BM-1, lo
// plane in BM..2BM-1 of the staged chunk) and WAVES * NT 16-column weight tiles; every wave keeps its NT
// weight fragments of a 128-element K step in registers (loaded straight from the tiled weights, two steps
// in flight) and all waves share the activation chunk, staged once per block in LDS (double buffered).
// The row blocks of one column tile re-read the same weights, so they are mapped to the SAME XCD and to
// adjacent dispatch slots: block id = xcd + 8 * (row block + n_mblocks * (tile / 8)); the re-reads then
// hit that XCD's L2 and HBM still sees every weight once.  The grid is padded to a multiple of 8 tiles.
template <int MODE, int BM, int KC, int NT, int WAVES, int NB>
__global__ __launch_bounds__(WAVES * 64) void gemm_tile_kernel(const uint16_t *A, ActView a_av,
                                                               WeightSeg w, int M, int N, int K, int k_per_split,
                                                               int n_mblocks, int n_ntiles, float *__restrict__ C,
                                                               size_t c_split_stride, uint16_t *__restrict__ Cact,
                                                               ActView c_av)
{
    constexpr int MT = BM / 16;      // 16-row tiles of A
    constexpr int OPROWS = 2 * BM;   // staged operand rows (hi | lo)
    constexpr int NI = KC / 32;      // MFMA k-groups per chunk (KC = 128: a whole K step, 64: half of one)
    static_assert(KC == 64 || KC == 128, "chunk is a K step or half of one");
    constexpr int LDROW = KC + GS_PAD;
    constexpr int THREADS = WAVES * 64;
    constexpr int VEC_PER_ROW = KC / 8; // 16-byte vectors per operand row
    constexpr int NVEC = OPROWS * VEC_PER_ROW;
    constexpr int LPT = NVEC / THREADS;
    static_assert(NVEC % THREADS == 0, "staging must divide evenly");
    constexpr bool SW = MODE == GEMM_SWIGLU;
    constexpr bool XCH = SW && (NT & 1); // gate/up pairs straddle waves
    static_assert(!SW || (NT * WAVES) % 2 == 0, "gate and up tiles come in pairs");
    constexpr int COLS = SW ? NT * WAVES * 8 : NT * 16 * WAVES; // output columns of a block
    __shared__ __attribute__((aligned(16))) uint16_t sA[2][OPROWS][LDROW];
    __shared__ f32x4 xch[XCH ? WAVES * MT * 64 : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = lane & 15, grp = lane >> 4;
    const int r8 = blockIdx.x >> 3;
    const int mblk = r8 % n_mblocks;
    const int ntile = (r8 / n_mblocks) * 8 + (blockIdx.x & 7);
    if (ntile >= n_ntiles) return; // padded grid
    const int n0 = ntile * COLS;
    const int m0 = mblk * BM;
    const int kb = blockIdx.y * k_per_split;
    const int ke = min(K, kb + k_per_split);
    const int nchunks = (ke - kb) / KC; // k_per_split and K are multiples of 128
    // this lane's 16 bytes inside the first K step of each of the wave's weight tiles
    const size_t tile_elems = (size_t)(K >> 7) * 2048;
    const uint16_t *Wp[NT];
    if (SW) {
        const int last_pair = N / 16 - 1; // pairs past the end (last block) re-read the last one; never stored
#pragma unroll
        for (int c = 0; c < NT; c++) {
            const int q = wave * NT + c;
            Wp[c] = (const uint16_t *)w.p[q & 1] + (size_t)min(n0 / 16 + (q >> 1), last_pair) * tile_elems +
                    (size_t)(kb >> 7) * 2048 + lane * 8;
        }
    } else {
        const int seg_tiles = w.n_per_seg / 16; // a block's tiles may lie in different segments (q | k | v)
#pragma unroll
        for (int c = 0; c < NT; c++) {
            const int tile = n0 / 16 + wave * NT + c;
            const int seg = tile / seg_tiles;
            const uint16_t *base = (const uint16_t *)(seg == 0 ? w.p[0] : seg == 1 ? w.p[1] : w.p[2]);
            Wp[c] = base + (size_t)(tile - seg * seg_tiles) * tile_elems + (size_t)(kb >> 7) * 2048 + lane * 8;
        }
    }
    // cooperative staging of the activation chunk: vector v -> operand row v / VEC_PER_ROW.  Rows past M
    // are loaded like any other (the buffers are over-allocated by SD_ACT_PAD_ROWS rows, so the addresses
    // are valid); whatever they hold only reaches accumulator rows that are never stored.
    uint32_t a_off[LPT];
    int a_dst[LPT];
#pragma unroll
    for (int j = 0; j < LPT; j++) {
        const int v = threadIdx.x + j * THREADS;
        const int orow = v / VEC_PER_ROW, ov = v % VEC_PER_ROW;
        a_off[j] = (uint32_t)((orow < BM ? 0 : a_av.plane) + (size_t)(m0 + orow % BM) * 128 + ov * 8);
        a_dst[j] = orow * LDROW + ov * 8;
    }
    const size_t step_stride = (size_t)a_av.rows * 128; // step-major activations
    // Loads for chunks past the end of the K range (issued by the last iterations so that every
    // iteration issues the same loads, which keeps the compiler's outstanding-load counts exact)
    // re-read the last chunk; their data is never used.
    bf16x8 a_reg[LPT];
    auto a_fetch = [&](int chunk) {
        const int k0 = min(chunk, nchunks - 1) * KC; // offset inside this block's K range
        const uint16_t *base = A + ((size_t)(kb >> 7) + (k0 >> 7)) * step_stride + (k0 & 127);
#pragma unroll
        for (int j = 0; j < LPT; j++) a_reg[j] = *(const bf16x8 *)(base + a_off[j]);
    };
    auto a_commit = [&](int buf) {
#pragma unroll
        for (int j = 0; j < LPT; j++) *(bf16x8 *)(&sA[buf][0][0] + a_dst[j]) = a_reg[j];
    };
    f32x4 acc[NT][MT];
#pragma unroll
    for (int c = 0; c < NT; c++)
#pragma unroll
        for (int t = 0; t < MT; t++) acc[c][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    bf16x8 wv[NB][NT][NI];
    auto w_issue = [&](int chunk, int b) {
        const int cc = min(chunk, nchunks - 1);
#pragma unroll
        for (int c = 0; c < NT; c++)
#pragma unroll
            for (int i = 0; i < NI; i++) wv[b][c][i] = *(const bf16x8 *)(Wp[c] + ((size_t)cc * NI + i) * 512);
    };
    // Activation fragments: two register sets used alternately by the MFMA groups of a chunk (group i
    // contracts elements 32*i .. 32*i+31 and reads set i & 1); the fragments of group i+1 are read from LDS
    // while group i runs.
    static_assert(NI % 2 == 0, "the last MFMA group of a chunk uses fragment set 1");
    bf16x8 fh[2][MT], fl[2][MT];
    auto frags = [&](int lb, int i, int fb) {
        const uint16_t *sa = &sA[lb][0][0] + row * LDROW + grp * 8;
#pragma unroll
        for (int t = 0; t < MT; t++) {
            fh[fb][t] = *(const bf16x8 *)(sa + t * 16 * LDROW + i * 32);
            fl[fb][t] = *(const bf16x8 *)(sa + (BM + t * 16) * LDROW + i * 32);
        }
    };
    auto mfma_group = [&](int b, int i) {
#pragma unroll
        for (int t = 0; t < MT; t++) {
#pragma unroll
            for (int c = 0; c < NT; c++)
                acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[b][c][i], fh[i & 1][t], acc[c][t], 0, 0, 0);
#pragma unroll
            for (int c = 0; c < NT; c++)
                acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[b][c][i], fl[i & 1][t], acc[c][t], 0, 0, 0);
        }
    };
    // Pipeline, iteration ch (weight buffer b = ch % NB):
    //   1. the activation rows of chunk ch+1 (fetched into registers during iteration ch-1) go to the
    //      other LDS buffer;
    //   2. chunk ch is multiplied, and in between its MFMAs the loads of later chunks are issued: the
    //      activation rows of chunk ch+2 first, then the weights of chunk ch+NB-1 into the buffer that
    //      iteration ch-1 released (so NB-1 weight chunks are in flight or in use at any time);
    //   3. barrier.  With EARLY the barrier stands before the last MFMA group instead, and the first
    //      fragments of chunk ch+1 are read from LDS behind it, under that group's MFMAs: no MFMA then
    //      waits for the LDS round trip that follows a barrier (it costs 8 more registers of live range,
    //      which only the 3-tile shape has to spare).
    // Every iteration issues the same loads in the same order, activation rows before weights: waiting
    // for the rows never waits for the (much slower) weight stream, and the wait counts stay exact.
    constexpr bool EARLY = BM == 96 && NT == 3;
    a_fetch(0);
    SD_ORDER();
    w_issue(0, 0);
    SD_ORDER();
    a_commit(0);
    a_fetch(1);
    SD_ORDER();
#pragma unroll
    for (int b = 1; b < NB - 1; b++) w_issue(b, b);
    SD_ORDER();
    __syncthreads();
    if (EARLY) {
        frags(0, 0, 0);
        SD_ORDER();
    }
    auto chunk = [&](int ch, int b) {
        a_commit((ch + 1) & 1);
        SD_ORDER();
        a_fetch(ch + 2);
        w_issue(ch + NB - 1, (b + NB - 1) % NB);
        if (!EARLY) frags(ch & 1, 0, 0);
#pragma unroll
        for (int i = 0; i < (EARLY ? NI - 1 : NI); i++) {
            if (i < NI - 1) frags(ch & 1, i + 1, (i + 1) & 1);
            mfma_group(b, i);
        }
        // instruction order of this stretch: (the LDS reads of the first fragment group, then) one
        // global load (activation rows first) and one LDS read after every third MFMA
        if (!EARLY) __builtin_amdgcn_sched_group_barrier(0x100, 2 * MT, 0);
#pragma unroll
        for (int k = 0; k < (NT * MT * 2 * (EARLY ? NI - 1 : NI)) / 3; k++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 3, 0); // MFMA
            if (k < LPT + NT * NI) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);     // VMEM read
            if (k < 2 * MT * (NI - 1)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); // DS read
        }
        SD_ORDER();
        __syncthreads();
        if (EARLY) {
            frags((ch + 1) & 1, 0, 0); // (after the last chunk: a stale buffer, never used)
            mfma_group(b, NI - 1);
#pragma unroll
            for (int k = 0; k < (NT * MT * 2) / 3; k++) {
                __builtin_amdgcn_sched_group_barrier(0x008, 3, 0); // MFMA
                if (k < 2 * MT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); // DS read
            }
            SD_ORDER();
        }
    };
    // whole rounds of NB chunks in one loop with a single exit (exits inside the unrolled round make the register
    // allocator copy accumulators from round to round), then the at most NB - 1 chunks that remain
    const int n_main = nchunks / NB * NB;
    for (int ch0 = 0; ch0 < n_main; ch0 += NB) {
#pragma unroll
        for (int b = 0; b < NB; b++) chunk(ch0 + b, b);
    }
#pragma unroll
    for (int b = 0; b < NB - 1; b++)
        if (n_main + b < nchunks) chunk(n_main + b, b);
    // epilogue: lane (m' = row, grp) holds D[n = 4*grp + r][m'] of each of its tiles
    f32x4 gin[MT]; // gate accumulators of the pair whose up tile is this wave's first tile
#pragma unroll
    for (int t = 0; t < MT; t++) gin[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (XCH) { // xch is used nowhere else; every wave is past the loop's last barrier
        if (((wave * NT + NT - 1) & 1) == 0) {
#pragma unroll
            for (int t = 0; t < MT; t++) xch[(wave * MT + t) * 64 + lane] = acc[NT - 1][t];
        }
        __syncthreads();
        if ((wave * NT) & 1) {
#pragma unroll
            for (int t = 0; t < MT; t++) gin[t] = xch[((wave - 1) * MT + t) * 64 + lane];
        }
    }
#pragma unroll
    for (int t = 0; t < MT; t++) {
        const int m = m0 + t * 16 + row;
        if (m >= M) continue;
        if (SW) {
#pragma unroll
            for (int c = 0; c < NT; c++) { // the wave that holds a pair's up tile writes the pair
                const int q = wave * NT + c;
                const int n = n0 + (q >> 1) * 16;
                if (!(q & 1) || n >= N) continue;
                const f32x4 g = c > 0 ? acc[c > 0 ? c - 1 : 0][t] : gin[t];
                const size_t o = act_index(c_av, m, n + 4 * grp, N); // 4 columns inside one K step: contiguous
                float y[4];
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const float g0 = g[r];
                    y[r] = g0 / (1.0f + expf(-g0)) * acc[c][t][r];
                }
                uint32_t h0, l0, h1, l1;
                bf16x2_split(y[0], y[1], h0, l0);
                bf16x2_split(y[2], y[3], h1, l1);
                *(uint2 *)(Cact + o) = make_uint2(h0, h1);
                *(uint2 *)(Cact + c_av.plane + o) = make_uint2(l0, l1);
            }
        } else {
            float *Cs = C + (size_t)blockIdx.y * c_split_stride;
#pragma unroll
            for (int c = 0; c < NT; c++) {
                const size_t o = (size_t)m * N + n0 + (wave * NT + c) * 16 + 4 * grp;
                *(f32x4 *)(Cs + o) = acc[c][t];
            }
        }
    }
}

// K range per split (a multiple of 128) and the number of splits that actually results
static void split_geometry(int K, int ks, int *kps, int *ny)
{
    if (ks < 1) ks = 1;
    if (K < 128) K = 128;
    *kps = ((K / 128 + ks - 1) / ks) * 128;
    *ny = (K + *kps - 1) / *kps;
}

// Few-row GEMM with the K range split over the 4 waves of a block (and optionally over grid.y).
// A block owns NTW 16-column tiles of NMAT matrices: NMAT = 1 stores fp32 sums (one slab per grid.y
// split), NMAT = 2 is the gate/up pair of the same columns with the SwiGLU epilogue (silu(gate)*up needs
// complete sums, so there grid.y is 1).  The waves interleave the 128-element K steps, fetch their
// activation fragments straight from global memory (L2) - no barrier inside the K loop - and keep the
// loads of U steps in flight in registers; the four partial accumulators meet in LDS.
template <int NMAT, bool PACKED, int MT, int U, int NTW, bool NT_HINT, int WAVES = 4>
__global__ __launch_bounds__(WAVES * 64) void gemm_ksplit_kernel(const uint16_t *__restrict__ A, ActView a_av, WeightSeg w,
                                                          int M, int N, int K, int steps_per_split,
                                                          float *__restrict__ C, size_t c_split_stride,
                                                          uint16_t *__restrict__ Cact, ActView c_av, LmStats ls,
                                                          NormFold nf)
{
    constexpr int THREADS = WAVES * 64;
    constexpr int NW = NMAT * NTW; // weight tiles per wave and step
    __shared__ float red[WAVES][NW][MT][64][4];
    __shared__ float s_inv[32]; // consumer side of a split norm: 1 / rms of every output row
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = lane & 15, grp = lane >> 4;
    const int n0 = blockIdx.x * 16 * NTW;
    // tiled weights: step st of a tile starts 2048*st elements after the tile, instruction i of a step
    // 512*i after that; tile j of matrix c is Wp[c] + j * tile_elems
    const size_t tile_elems = (size_t)(K >> 7) * 2048;
    const uint16_t *Wp[NMAT];
    if (NMAT == 2) {
#pragma unroll
        for (int c = 0; c < NMAT; c++) Wp[c] = (const uint16_t *)w.p[c] + (size_t)(n0 / 16) * tile_elems + lane * 8;
    } else {
        const int seg = n0 / w.n_per_seg;
        Wp[0] = (const uint16_t *)w.p[seg] + (size_t)((n0 - seg * w.n_per_seg) / 16) * tile_elems + lane * 8;
    }
    const uint16_t *Ap[MT], *Al[MT];
    bool a_live[MT];
#pragma unroll
    for (int t = 0; t < MT; t++) {
        const int m = PACKED ? (row & 7) : t * 16 + row;
        a_live[t] = m < M;
        const int src = !a_live[t] ? 0 : nf.row_map ? nf.row_map[m] : m;
        // step-major activations: row m of K step st starts at (st * rows + m) * 128
        Ap[t] = A + ((PACKED && row >= 8) ? a_av.plane : 0) + (size_t)src * 128 + grp * 8;
        Al[t] = Ap[t] + a_av.plane;
    }
    constexpr int ROWS_MAX = PACKED ? 8 : 16 * MT;
    constexpr int SSR = (ROWS_MAX + WAVES - 1) / WAVES, SSB = SD_NORMFOLD_MAX_BLOCKS / 256; // (a lane loads 4 entries at once)
    constexpr int EPI = (16 * NTW * ROWS_MAX + THREADS - 1) / THREADS; // epilogue elements per thread
    float4 ssl[SSR][SSB]; // consumer side of a split norm: wave w sums the producer's per-block shares of rows w, w + 4, ...
    int ss_src[SSR];
    float xres[EPI], gval[EPI]; // producer side: residual and gain of this thread's epilogue elements
    if (nf.ss_in) {
#pragma unroll
        for (int r = 0; r < SSR; r++) {
            const int m = wave + r * WAVES;
            ss_src[r] = m < M ? (nf.row_map ? nf.row_map[m] : m) : 0;
        }
    }
    const size_t step_stride = (size_t)a_av.rows * 128;
    f32x4 acc[NW][MT];
#pragma unroll
    for (int c = 0; c < NW; c++)
#pragma unroll
        for (int t = 0; t < MT; t++) acc[c][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const int s_begin = blockIdx.y * steps_per_split;
    const int s_end = min(K / 128, s_begin + steps_per_split);
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    // U register buffers: the loads of the wave's next U-1 steps are in flight while one step is consumed
    bf16x8 wv[U][NW][4], av[U][MT][4], al[U][PACKED ? 1 : MT][4];
    auto issue = [&](int st, int b) {
#pragma unroll
        for (int t = 0; t < MT; t++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                av[b][t][i] = a_live[t] ? *(const bf16x8 *)(Ap[t] + step_stride * st + i * 32) : zero;
                if (!PACKED) al[b][t][i] = a_live[t] ? *(const bf16x8 *)(Al[t] + step_stride * st + i * 32) : zero;
            }
#pragma unroll
        for (int c = 0; c < NW; c++)
#pragma unroll
            for (int i = 0; i < 4; i++)
                wv[b][c][i] = ld_stream<NT_HINT>((const bf16x8 *)(Wp[c % NMAT] + (size_t)(c / NMAT) * tile_elems + (size_t)st * 2048 + i * 512));
    };
    // the small loads of a split norm go out ahead of the weight stream (loads return in order: behind the
    // first weight loads they would hold up everything issued after them for as long as they take) and are used
    // after the K loop; every address is clamped into range, so the loads are unconditional
    if (nf.ss_in) { // (uniform)
#pragma unroll
        for (int r = 0; r < SSR; r++)
#pragma unroll
            for (int i = 0; i < SSB; i++) // (entries past ss_nb are stale or never written: masked when summed)
                ssl[r][i] = *(const float4 *)(nf.ss_in + ss_src[r] * SD_NORMFOLD_MAX_BLOCKS + 4 * (lane + 64 * i));
    }
    if (NMAT == 1 && nf.x) { // (uniform)
#pragma unroll
        for (int k = 0; k < EPI; k++) {
            const int e = threadIdx.x + THREADS * k;
            const int m = min(e / (16 * NTW), M - 1), n = n0 + (e & (16 * NTW - 1));
            xres[k] = nf.x[(size_t)m * N + n];
            gval[k] = nf.g[n];
        }
    }
#pragma unroll
    for (int u = 0; u < U; u++)
        if (s_begin + wave + u * WAVES < s_end) issue(s_begin + wave + u * WAVES, u);
    // The wave's rows of 1 / rms: summed once its first K step has been consumed - the small loads went out
    // before that step's and have therefore arrived - so that nothing of it is left for the block's tail.
    bool ss_pending = nf.ss_in != nullptr;
    auto ss_reduce = [&]() {
#pragma unroll
        for (int r = 0; r < SSR; r++) {
            float a = 0.f;
#pragma unroll
            for (int i = 0; i < SSB; i++) {
                const int b = 4 * (lane + 64 * i);
                a += b < nf.ss_nb ? ssl[r][i].x : 0.f;
                a += b + 1 < nf.ss_nb ? ssl[r][i].y : 0.f;
                a += b + 2 < nf.ss_nb ? ssl[r][i].z : 0.f;
                a += b + 3 < nf.ss_nb ? ssl[r][i].w : 0.f;
            }
            a = wave_sum_dpp(a);
            const int m = wave + r * WAVES;
            if (lane == 0 && m < ROWS_MAX) s_inv[m] = 1.0f / sqrtf(a / (float)K + nf.eps);
        }
        ss_pending = false;
    };
    for (int s = s_begin + wave; s < s_end; s += U * WAVES) {
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int cur = s + u * WAVES;
            if (cur < s_end) {
#pragma unroll
                for (int i = 0; i < 4; i++)
#pragma unroll
                    for (int t = 0; t < MT; t++)
#pragma unroll
                        for (int c = 0; c < NW; c++) {
                            acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[u][c][i], av[u][t][i], acc[c][t], 0, 0, 0);
                            if (!PACKED)
                                acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[u][c][i], al[u][t][i], acc[c][t], 0, 0, 0);
                        }
                if (cur + U * WAVES < s_end) issue(cur + U * WAVES, u);
                if (u == 0 && ss_pending) ss_reduce(); // (uniform; true in the first round only)
            }
        }
    }
#pragma unroll
    for (int c = 0; c < NW; c++)
#pragma unroll
        for (int t = 0; t < MT; t++)
#pragma unroll
            for (int r = 0; r < 4; r++) red[wave][c][t][lane][r] = acc[c][t][r];
    if (ss_pending) ss_reduce(); // (a wave without a K step of its own)
    __syncthreads();
    // tile element D[n = 4*(slot/16) + r][m' = slot%16] sits at red[.][c][t][slot][r]
    constexpr int ROWS = PACKED ? 8 : 16 * MT;
    for (int e = threadIdx.x, ek = 0; e < 16 * NTW * ROWS; e += THREADS, ek++) {
        const int nn = e & 15, j = (e >> 4) % NTW, m = e / (16 * NTW);
        if (m >= M) continue;
        const int t = PACKED ? 0 : m >> 4;
        const int slot = (nn >> 2) * 16 + (m & 15), r = nn & 3;
        float v[NMAT];
#pragma unroll
        for (int c = 0; c < NMAT; c++) {
            v[c] = 0.f;
#pragma unroll
            for (int wv2 = 0; wv2 < WAVES; wv2++) {
                v[c] += red[wv2][j * NMAT + c][t][slot][r];
                if (PACKED) v[c] += red[wv2][j * NMAT + c][t][slot + 8][r];
            }
            if (nf.ss_in) v[c] *= s_inv[m];
        }
        if (NMAT == 1 && nf.x) { // (uniform) producer side of a split norm; the launcher rules out K splits
            const int n = n0 + j * 16 + nn;
            float xr = xres[0], gg = gval[0];
#pragma unroll
            for (int k = 1; k < EPI; k++)
                if (k == ek) xr = xres[k], gg = gval[k];
            const float xn = xr + v[0];
            nf.x[(size_t)m * N + n] = xn;
            const float y = xn * gg;
            const uint16_t hi = bf16_bits_rne(y);
            const size_t o = act_index(c_av, m, n, N);
            Cact[o] = hi;
            Cact[c_av.plane + o] = bf16_bits_rne(y - __uint_as_float((uint32_t)hi << 16));
            float sq = row16_sum(xn * xn); // the block's 16 * NTW columns of row m sit in adjacent lanes
            if (NTW == 2) sq += __shfl_xor(sq, 16, 64);
            if ((e & (16 * NTW - 1)) == 0) nf.ss_out[m * SD_NORMFOLD_MAX_BLOCKS + blockIdx.x] = sq;
            continue;
        }
        if (NMAT == 2) {
            const float y = v[0] / (1.0f + expf(-v[0])) * v[NMAT - 1];
            const uint16_t hi = bf16_bits_rne(y);
            const size_t o = act_index(c_av, m, n0 + j * 16 + nn, N);
            Cact[o] = hi;
            Cact[c_av.plane + o] = bf16_bits_rne(y - __uint_as_float((uint32_t)hi << 16));
        } else {
            C[(size_t)blockIdx.y * c_split_stride + (size_t)m * N + n0 + j * 16 + nn] = v[0];
            if (NTW == 2 && ls.p) { // (uniform) the block's 32 columns of row m sit in the 32 lanes of a half wave
                float mx = v[0];
                int ai = n0 + j * 16 + nn;
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) {
                    const float ov = __shfl_xor(mx, o, 64);
                    const int oi = __shfl_xor(ai, o, 64);
                    if (ov > mx || (ov == mx && oi < ai)) {
                        mx = ov;
                        ai = oi;
                    }
                }
                float ex = ls.invT > 0.f ? expf((v[0] - mx) * ls.invT) : 0.f;
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) ex += __shfl_xor(ex, o, 64);
                if ((e & 31) == 0) {
                    float *sp = ls.p + ((size_t)m * gridDim.x + blockIdx.x) * 3;
                    sp[0] = mx;
                    sp[1] = ex;
                    sp[2] = __int_as_float(ai);
                }
            }
        }
    }
}

// Block shapes of the row-blocked kernel.  More than 64 rows: 96 rows x 256 columns (4 waves x 4 tiles; chunks
// of half a K step) - the bytes a block pulls through L2 per MFMA halve against 48 x 128, which is what
// bounds these GEMMs - or x 192 columns (3 tiles per wave) where that fills the 256 compute units better
// (QKV at M = 192: 128 blocks x 2 K splits instead of 96 x 2); 64-row blocks of the same widths where they
// pad M less (M = 128).  Up to 64 rows: 48-row blocks of 2 waves x
// 128 columns, two resident per unit.  A block of the 96-row shapes has a compute unit to itself
// (~500 registers per wave), so the K splits are chosen to cover the chip in one round of blocks.
struct TileShape {
    int cols;  // weight rows per block (0: shape not supported)
    int bm;    // rows per block
    int ncol;  // column tiles
    int nmb;   // row blocks
    int slots; // blocks resident at once on the whole chip
};
// Column tile t runs on die t % 8 with all its row blocks and K splits (they share the die's L2), so the busiest
// die carries ceil(ncol / 8) tiles: 20 tiles put 3 on four dies and 2 on the others.  A launch is one round of
// blocks only if that die's share fits its eighth of the slots - counting blocks over the whole chip instead let
// the 5120-wide projections run a second round on half the dies (44 against 31 us for the O projection at M = 192).
static int die_blocks(int ncol, int nmb, int ks) { return (ncol + 7) / 8 * nmb * ks; }
static int one_round_splits(int ncol, int nmb, int slots, int steps)
{
    int ks = 1;
    while (ks < 8 && die_blocks(ncol, nmb, ks + 1) * 8 <= slots && (steps + ks) / (ks + 1) >= 4) ks++;
    return ks;
}
static int die_rounds(int ncol, int nmb, int ks, int slots) { return (die_blocks(ncol, nmb, ks) * 8 + slots - 1) / slots; }
// K splits of a launch: as many as keep the busiest die at one round of blocks; where not even the unsplit launch fits one
// round, the count that makes rounds x (K steps per split + 5 steps of fixed cost) smallest (by more than 5 %): the 96-row
// QKV blocks of a 4096-wide model at M = 576 come to one and a half rounds, two splits to three full ones of half the
// length (measured 120 -> 107 us; three and four splits 124 us, as the model has it).
static int tile_splits(int ncol, int nmb, int slots, int steps)
{
    if (die_rounds(ncol, nmb, 1, slots) == 1) return one_round_splits(ncol, nmb, slots, steps);
    int best = 1;
    float best_cost = (float)die_rounds(ncol, nmb, 1, slots) * ((float)steps + 5.f);
    for (int ks = 2; ks <= 8 && (steps + ks - 1) / ks >= 4; ks++) {
        const float cost = (float)die_rounds(ncol, nmb, ks, slots) * ((float)steps / (float)ks + 5.f);
        if (cost < 0.95f * best_cost) {
            best = ks;
            best_cost = cost;
        }
    }
    return best;
}
int g_force_tile_cols = 0; // weight rows per 96-row block forced by option "gemm_tile_cols" (0 = automatic)
static TileShape tile_shape(int mode, int M, int N, int n_per_seg, int K)
{
    const int out_per_col = mode == GEMM_SWIGLU ? 2 : 1; // weight rows per output column
    const int rows_w = N * out_per_col;                  // weight rows streamed
    TileShape t = {0, 0, 0, 0, 0};
    if (M > 64) {
        const int nmb = (M + 95) / 96, steps = K / 128;
        const bool ok256 = rows_w % 256 == 0 && (mode == GEMM_SWIGLU || n_per_seg % 256 == 0);
        // (SwiGLU blocks of 192 weight rows = 96 output columns may end in a partial block)
        const bool ok192 = mode == GEMM_SWIGLU || (rows_w % 192 == 0 && n_per_seg % 16 == 0);
        auto fill = [&](int cols) { // fraction of the 256 units busy, averaged over the rounds of blocks
            const int ncol = (rows_w + cols - 1) / cols;
            const int ks = mode == GEMM_SWIGLU ? 1 : one_round_splits(ncol, nmb, 256, steps);
            return (float)(ncol * nmb * ks) / (256.f * (float)die_rounds(ncol, nmb, ks, 256));
        };
        int cols = 0;
        if (ok256) cols = 256;
        if (ok192 && (!ok256 || fill(192) > fill(256) + 0.1f)) cols = 192;
        // Plain projections with few column tiles may do better with 128-column blocks.  A block's time is modelled as
        // rounds on the busiest die x (K steps per split + 5 steps of fixed cost) x the cost of one of its steps (a
        // 128-column step costs 0.68 of a 256-column one: half the weights and MFMAs, the same activation chunk).
        // Against measurements at widths 4096 and 5120, M = 66 ... 576, it picks 128 columns for O and down at M <= 96
        // (twice the blocks in flight), for O at M = 192 (4 K splits of 8 steps instead of 8 of 4: also half the slabs
        // for the add + norm launch behind it) and for the 5120-wide O and down where 20 wide tiles would leave four
        // dies with half as much again as the others; 256 columns for the 4096-wide down projection at M > 96 and for
        // QKV.
        const bool ok128 = mode != GEMM_SWIGLU && rows_w % 128 == 0 && n_per_seg % 128 == 0;
        if (cols == 256 && ok128) {
            auto est = [&](int c, float step_cost) {
                const int ncol = rows_w / c, sp = one_round_splits(ncol, nmb, 256, steps);
                return (float)die_rounds(ncol, nmb, sp, 256) * ((float)steps / (float)sp + 5.f) * step_cost;
            };
            if (est(128, 0.68f) < est(256, 1.f)) cols = 128;
        }
        if (g_force_tile_cols == 256 && ok256) cols = 256;
        if (g_force_tile_cols == 192 && ok192) cols = 192;
        if (g_force_tile_cols == 128 && ok128) cols = 128;
        if (cols) {
            // 64-row blocks when they pad M less (M = 128: 2 x 64 instead of 96 + 32) and do not cost more rounds
            const int ncol = (rows_w + cols - 1) / cols, nmb64 = (M + 63) / 64;
            auto rounds = [&](int rb) {
                return die_rounds(ncol, rb, mode == GEMM_SWIGLU ? 1 : one_round_splits(ncol, rb, 256, steps), 256);
            };
            const bool use64 = nmb64 * 64 < nmb * 96 && rounds(nmb64) * 64 <= rounds(nmb) * 96;
            return use64 ? TileShape{cols, 64, ncol, nmb64, 256} : TileShape{cols, 96, ncol, nmb, 256};
        }
    }
    if (rows_w % 128 == 0 && (mode == GEMM_SWIGLU || n_per_seg % 128 == 0))
        t = TileShape{128, 48, rows_w / 128, (M + 47) / 48, 512};
    return t;
}

template <int MODE>
static hipError_t tile_launch(hipStream_t s, const uint16_t *a, ActView a_av, WeightSeg w, int M, int N, int K, int ks,
                              float *C, size_t c_split_stride, uint16_t *ca, ActView c_av)
{
    int kps, ny;
    split_geometry(K, ks, &kps, &ny);
    const TileShape t = tile_shape(MODE, M, N, w.n_per_seg, K);
    if (!t.cols) return hipErrorNotSupported;
    constexpr int OUT_PER_COL = MODE == GEMM_SWIGLU ? 2 : 1;
    const int ntiles = (N * OUT_PER_COL + t.cols - 1) / t.cols, nmb = (M + t.bm - 1) / t.bm;
    const int gx = ((ntiles + 7) / 8) * 8 * nmb;
#define SD_TILE(BM, KC, NT, WAVES, NB)                                                                              \
    hipLaunchKernelGGL((gemm_tile_kernel<MODE, BM, KC, NT, WAVES, NB>), dim3(gx, ny), dim3(WAVES * 64), 0, s, a, a_av, w, \
                       M, N, K, kps, nmb, ntiles, C, c_split_stride, ca, c_av)
    if (t.cols == 256 && t.bm == 96) SD_TILE(96, 64, 4, 4, 3);
    else if (t.cols == 192 && t.bm == 96) SD_TILE(96, 64, 3, 4, 3);
    else if (t.cols == 256) SD_TILE(64, 64, 4, 4, 3);
    else if (t.cols == 192) SD_TILE(64, 64, 3, 4, 3);
    else if (t.cols == 128 && t.bm == 96) SD_TILE(96, 64, 2, 4, 3);
    else if (t.cols == 128 && t.bm == 64) SD_TILE(64, 64, 2, 4, 3);
    else SD_TILE(48, 128, 4, 2, 3);
    return hipGetLastError();
}

int g_force_splits[3] = {0, 0, 0}; // [mode] -> K splits (0 = automatic); a tuning knob for sweeps

// Number of K splits the launcher will use for this shape (the caller sizes and reduces the partials).
int gemm_skinny_splits(int mode, int M, int N, int K, int n_per_seg)
{
    if (mode == GEMM_SWIGLU || K < 128 || K % 128 != 0) return 1; // (the launcher rejects such K)
    int kps, ny;
    if (g_force_splits[mode] > 0) {
        split_geometry(K, g_force_splits[mode], &kps, &ny);
        return ny;
    }
    const int steps = K / 128;
    int ks;
    if (M <= 32) { // K-split kernel: 32 columns per block, each wave at least 2 steps
        const int blocks = N / 32;
        ks = steps >= 16 ? 2 : 1; // measured: two half-length blocks per tile stream faster than one
        while (blocks * ks < 256 && ks < 8 && steps / (ks * 2) >= 4) ks *= 2;
    } else { // row-blocked kernel.  Measured at M = 192: a block costs about five K steps of fixed time, so one
             // round of blocks with the K range cut as finely as that allows beats several rounds of shorter blocks
        const TileShape t = tile_shape(mode, M, N, n_per_seg, K);
        ks = t.cols ? tile_splits(t.ncol, t.nmb, t.slots, steps) : 1;
    }
    split_geometry(K, ks, &kps, &ny);
    return ny;
}

// What tile_launch would do for this shape (host only; for tests of the choice itself).
int gemm_tile_plan(int mode, int M, int N, int K, int n_per_seg, int plan[6])
{
    if (M <= 32 || K < 128 || K % 128 != 0 || (mode != GEMM_STORE && mode != GEMM_SWIGLU)) return -1;
    const TileShape t = tile_shape(mode, M, N, n_per_seg, K);
    if (!t.cols) return -1;
    const int ks = gemm_skinny_splits(mode, M, N, K, n_per_seg);
    plan[0] = t.cols;
    plan[1] = t.bm;
    plan[2] = t.ncol;
    plan[3] = t.nmb;
    plan[4] = ks;
    plan[5] = die_blocks(t.ncol, t.nmb, ks);
    return 0;
}

// Blocks (= entries of NormFold::ss_out per row) of a producer launch with N output columns.
int gemm_normfold_blocks(int N) { return N % 32 == 0 && N / 32 >= 256 ? N / 32 : N / 16; }

// mode GEMM_STORE: C receives `splits` partial slabs [split][M][N] (split stride c_split_stride floats);
// mode GEMM_SWIGLU: Cact receives the bf16 hi/lo planes.  GEMM_RESID is expressed by the caller as a
// store into partial slabs followed by the fused add + norm kernel.
hipError_t launch_gemm_skinny_bf16(hipStream_t s, int mode, const void *A, ActView a_av, WeightSeg w, int M, int N,
                                   int K, float *C, size_t c_split_stride, int splits, void *Cact, ActView c_av,
                                   LmStats ls, int *ls_done, NormFold nf)
{
    if (ls_done) *ls_done = 0;
    const LmStats no_ls = {nullptr, 0.f};
    const bool folded = nf.ss_in || nf.x || nf.row_map;
    if (folded && (M > 32 || nf.ss_nb > SD_NORMFOLD_MAX_BLOCKS)) return hipErrorNotSupported;
    if (nf.x && (mode != GEMM_STORE || splits != 1 || !c_av.sm || N % 128 != 0 || N / 16 > SD_NORMFOLD_MAX_BLOCKS))
        return hipErrorNotSupported;
    if (M < 1 || K % 128 != 0 || K < 128 || (mode != GEMM_STORE && mode != GEMM_SWIGLU)) return hipErrorNotSupported;
    if (!w.tiled) return hipErrorNotSupported; // these kernels read the 16 x 128 tile order only
    for (int i = 0; i < 3; i++)
        if (w.p[i] && ((uintptr_t)w.p[i] & 15)) return hipErrorNotSupported;
    if (((uintptr_t)A & 15) || (a_av.plane & 7) || (N & 3) || !a_av.sm || a_av.rows < M) return hipErrorNotSupported;
    if (2 * a_av.plane + (size_t)SD_ACT_PAD_ROWS * 128 >= ((size_t)1 << 32)) return hipErrorNotSupported; // 32-bit offsets
    if (mode == GEMM_SWIGLU && (!c_av.sm || (c_av.plane & 7) || N % 128 != 0 || ((uintptr_t)Cact & 15))) return hipErrorNotSupported;
    const uint16_t *a = (const uint16_t *)A;
    uint16_t *ca = (uint16_t *)Cact;
    if (M > 32) { // row-blocked
        if (mode == GEMM_SWIGLU) return tile_launch<GEMM_SWIGLU>(s, a, a_av, w, M, N, K, 1, C, 0, ca, c_av);
        return tile_launch<GEMM_STORE>(s, a, a_av, w, M, N, K, splits, C, c_split_stride, ca, c_av);
    }
#define SD_KSPLIT(NMAT, PACKED, MT, U, NTW, GRID, SPS, LS)                                                               \
    do {                                                                                                                  \
        if (w.nt)                                                                                                         \
            hipLaunchKernelGGL((gemm_ksplit_kernel<NMAT, PACKED, MT, U, NTW, true>), GRID, dim3(256), 0, s, a, a_av, w, M, \
                               N, K, SPS, C, c_split_stride, ca, c_av, LS, nf);                                           \
        else                                                                                                              \
            hipLaunchKernelGGL((gemm_ksplit_kernel<NMAT, PACKED, MT, U, NTW, false>), GRID, dim3(256), 0, s, a, a_av, w,  \
                               M, N, K, SPS, C, c_split_stride, ca, c_av, LS, nf);                                        \
    } while (0)
    if (mode == GEMM_SWIGLU) { // K split inside the block only
        if (N % 16 != 0) return hipErrorNotSupported;
        dim3 grid(N / 16);
        if (M <= 8) SD_KSPLIT(2, true, 1, 2, 1, grid, K / 128, no_ls);
        else if (M <= 16) SD_KSPLIT(2, false, 1, 2, 1, grid, K / 128, no_ls);
        else SD_KSPLIT(2, false, 2, 1, 1, grid, K / 128, no_ls);
        return hipGetLastError();
    }
    int kps, ny;
    split_geometry(K, splits, &kps, &ny);
    if (nf.x && ny != 1) return hipErrorNotSupported;
    // (a producer of a split norm has no K split to fill the chip with: 16-column blocks where 32-column ones would
    // leave compute units idle, and four K steps in flight per wave instead of two)
    if (N % 32 == 0 && w.n_per_seg % 32 == 0 && !(nf.x && N / 32 < 256)) {
        dim3 grid(N / 32, ny);
        const LmStats lsk = ny == 1 ? ls : no_ls; // (partial sums of a K split have no softmax)
        if (ls_done && lsk.p) *ls_done = 1;
        if (M <= 8) SD_KSPLIT(1, true, 1, 2, 2, grid, kps / 128, lsk);
        else if (M <= 16) SD_KSPLIT(1, false, 1, 2, 2, grid, kps / 128, lsk);
        else SD_KSPLIT(1, false, 2, 1, 2, grid, kps / 128, lsk);
    } else if (N % 16 == 0 && w.n_per_seg % 16 == 0) {
        dim3 grid(N / 16, ny);
        if (M <= 8 && nf.x) SD_KSPLIT(1, true, 1, 4, 1, grid, kps / 128, no_ls);
        else if (M <= 8) SD_KSPLIT(1, true, 1, 2, 1, grid, kps / 128, no_ls);
        else if (M <= 16) SD_KSPLIT(1, false, 1, 2, 1, grid, kps / 128, no_ls);
        else SD_KSPLIT(1, false, 2, 1, 1, grid, kps / 128, no_ls);
    } else {
        return hipErrorNotSupported;
    }
    return hipGetLastError();
}
