// bf16 weight-streaming GEMM for few rows (M <= 32): C[M][N] = A[M][K] . W[N][K]^T.
//
// This is the verify forward at batch 1 (M = gamma+1) and every draft step: the
// work is reading each weight once from HBM, so the kernel is organised around
// the weight stream, and the matrix cores only keep the ALUs out of the way.
//
//  * a block of WAVES waves covers WAVES*16*NT/... output columns and one K range
//    (grid.y splits K); every wave owns NT 16-column tiles of W and all waves walk
//    the same K chunks, so the activation chunk is staged ONCE per block in LDS
//    (double buffered) instead of being fetched by every wave from L2 - at these
//    sizes the shared activation lines, not HBM, were the bottleneck otherwise;
//  * weights are stored in 16-row x 128-element tiles in MFMA operand order, so each
//    of the four load instructions of a K step reads one contiguous kilobyte straight
//    into operand registers (v_mfma_f32_16x16x32_bf16: lane l supplies row l%16,
//    k-group l/16), all steps of a chunk in flight at once.  Row-major weights would
//    spread every such load over 16 rows 2K bytes apart, which lands on one L2 channel
//    and limits a compute unit to about a third of the rate it reaches on the tiles;
//  * activations are two bf16 planes (hi + lo, ~16 mantissa bits).  For M <= 8 both
//    planes ride in ONE operand: MFMA columns 0..7 carry the hi rows, columns 8..15
//    the lo rows, and the epilogue adds the two halves with one lane exchange; for
//    larger M every weight fragment is multiplied twice;
//  * results leave either directly (store; SwiGLU: silu(gate)*up split to bf16
//    hi/lo) or as fp32 partial sums per K split, which the consuming kernel adds in
//    a fixed order (rope_append for QKV, add_rmsnorm for the residual GEMMs), so
//    results are bit-reproducible run to run.
//
// Paper (arXiv 2505.08600): Section 1, Figure 1 (draft steps and the parallel
// verify pass whose linear layers these are); Section 3.1 (LLaMA blocks).
#include "sd_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define GS_OPELEMS 8192 // bf16 elements of one staged activation chunk (operand rows x chunk length)
#define GS_PAD 8        // row padding in LDS (16 bytes): operand rows fall into distinct banks

// MODE: GEMM_STORE (C = acc, or partial sums when KS > 1) / GEMM_SWIGLU (tiles 2j, 2j+1 of a wave are
// the gate and up tile of the same columns).  OPROWS: operand rows staged per chunk: 16 (packed hi|lo,
// M <= 8), 32 (hi 0..15, lo 16..31, M <= 16) or 64 (M <= 32).
// For M > 32 the rows are cut into blocks of OPROWS/2 = 48 rows (n_mblocks >= 1 of them; n_mblocks == 0
// selects the plain mapping block = column tile, with an exact grid); the row blocks of
// one column tile re-read the same weights, so they are mapped to the SAME XCD and to adjacent dispatch
// slots: the re-reads then hit that XCD's L2 and HBM still sees every weight once.
template <int MODE, int OPROWS, int KC, int NT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemm_stream_kernel(const uint16_t *__restrict__ A, size_t a_plane,
                                                                 WeightSeg w, int M, int N, int K, int k_per_split,
                                                                 int n_mblocks, int n_ntiles,
                                                                 float *__restrict__ C, size_t c_split_stride,
                                                                 uint16_t *__restrict__ Cact, size_t c_plane)
{
    constexpr bool PACKED = OPROWS == 16;
    constexpr int MT = PACKED ? 1 : OPROWS / 32;    // 16-row tiles of A
    constexpr int BM = PACKED ? 8 : OPROWS / 2;     // rows of A per block
    constexpr int STEPS = KC / 128;                 // 128-element steps per chunk
    constexpr int LDROW = KC + GS_PAD;
    constexpr int THREADS = WAVES * 64;
    constexpr int VEC_PER_ROW = KC / 8;             // 16-byte vectors per operand row
    constexpr int NVEC = OPROWS * VEC_PER_ROW;      // vectors per chunk
    constexpr int LPT = (NVEC + THREADS - 1) / THREADS;
    constexpr int COLS = (MODE == GEMM_SWIGLU ? NT / 2 : NT) * 16 * WAVES;
    __shared__ __attribute__((aligned(16))) uint16_t sA[2][OPROWS][LDROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = lane & 15, grp = lane >> 4;
    // block -> (column tile, row block): id = xcd + 8 * (row block + n_mblocks * (tile / 8))
    int ntile = blockIdx.x, mblk = 0;
    if (n_mblocks >= 1) { // row-blocked launch: the grid is padded, so the tile index must be checked
        const int r = blockIdx.x >> 3;
        mblk = r % n_mblocks;
        ntile = (r / n_mblocks) * 8 + (blockIdx.x & 7);
        if (ntile >= n_ntiles) return; // grid is padded to a multiple of 8 tiles
    }
    const int n0 = ntile * COLS;
    const int m0 = mblk * BM;
    const int kb = blockIdx.y * k_per_split;
    const int ke = min(K, kb + k_per_split);
    const int nchunks = (ke - kb + KC - 1) / KC;
    // this lane's 16 bytes inside the first K step of each of the wave's 16-row weight tiles (tiled order:
    // a tile's steps are 2048 elements apart, the four load instructions of a step 512 elements)
    const size_t tile_elems = (size_t)(K >> 7) * 2048;
    const uint16_t *Wp[NT];
    if (MODE == GEMM_SWIGLU) {
#pragma unroll
        for (int c = 0; c < NT; c++)
            Wp[c] = (const uint16_t *)w.p[c & 1] + (size_t)(n0 / 16 + wave * (NT / 2) + (c >> 1)) * tile_elems + lane * 8;
    } else {
        const int seg = n0 / w.n_per_seg;
        const int nl = n0 - seg * w.n_per_seg;
#pragma unroll
        for (int c = 0; c < NT; c++)
            Wp[c] = (const uint16_t *)w.p[seg] + (size_t)(nl / 16 + wave * NT + c) * tile_elems + lane * 8;
    }
    // cooperative staging of the activation chunk: vector v -> operand row v / VEC_PER_ROW
    const uint16_t *a_src[LPT];
    int a_dst[LPT];
    bool a_ok[LPT];
#pragma unroll
    for (int j = 0; j < LPT; j++) {
        const int v = threadIdx.x + j * THREADS;
        const int orow = v / VEC_PER_ROW, ov = v % VEC_PER_ROW;
        int m;
        size_t plane;
        if (PACKED) {
            m = orow & 7;
            plane = orow < 8 ? 0 : a_plane;
        } else {
            m = m0 + (orow % (OPROWS / 2));
            plane = orow < OPROWS / 2 ? 0 : a_plane;
        }
        a_ok[j] = v < NVEC && m < M;
        a_src[j] = A + plane + (size_t)(a_ok[j] ? m : 0) * K + ov * 8;
        a_dst[j] = (v < NVEC ? orow : 0) * LDROW + ov * 8;
    }
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    bf16x8 a_reg[LPT];
    auto a_fetch = [&](int chunk) {
        const int k0 = kb + chunk * KC;
#pragma unroll
        for (int j = 0; j < LPT; j++) {
            const int ov8 = (a_dst[j] % LDROW);
            a_reg[j] = (a_ok[j] && k0 + ov8 < ke) ? *(const bf16x8 *)(a_src[j] + k0) : zero;
        }
    };
    auto a_commit = [&](int buf) {
#pragma unroll
        for (int j = 0; j < LPT; j++)
            if (threadIdx.x + j * THREADS < NVEC) *(bf16x8 *)(&sA[buf][0][0] + a_dst[j]) = a_reg[j];
    };
    f32x4 acc[NT][MT];
#pragma unroll
    for (int c = 0; c < NT; c++)
#pragma unroll
        for (int t = 0; t < MT; t++) acc[c][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // Weight loads of a chunk: all steps in flight at once.  They are issued for chunk ch+1 right after
    // the MFMAs of chunk ch released the registers, i.e. before the barrier, so HBM never waits on LDS.
    bf16x8 wv[NT][STEPS][4];
    auto w_issue = [&](int chunk) {
        const int k0 = kb + chunk * KC;
#pragma unroll
        for (int c = 0; c < NT; c++)
#pragma unroll
            for (int st = 0; st < STEPS; st++) {
                const int k = k0 + st * 128;
                const bool live = k < ke;
                const uint16_t *p = Wp[c] + (size_t)((live ? k : kb) >> 7) * 2048;
#pragma unroll
                for (int i = 0; i < 4; i++) wv[c][st][i] = live ? *(const bf16x8 *)(p + i * 512) : zero;
            }
    };
    w_issue(0);
    a_fetch(0);
    a_commit(0);
    __syncthreads();
    for (int ch = 0; ch < nchunks; ch++) {
        const bool more = ch + 1 < nchunks;
        if (more) a_fetch(ch + 1);
        const uint16_t *sa = &sA[ch & 1][0][0];
#pragma unroll
        for (int st = 0; st < STEPS; st++) {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int kk = st * 128 + i * 32 + grp * 8; // MFMA i contracts elements 32*i .. 32*i+31 of the step
#pragma unroll
                for (int t = 0; t < MT; t++) {
                    if (PACKED) {
                        const bf16x8 av = *(const bf16x8 *)(sa + row * LDROW + kk);
#pragma unroll
                        for (int c = 0; c < NT; c++)
                            acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[c][st][i], av, acc[c][t], 0, 0, 0);
                    } else {
                        const bf16x8 ah = *(const bf16x8 *)(sa + (t * 16 + row) * LDROW + kk);
                        const bf16x8 al = *(const bf16x8 *)(sa + (OPROWS / 2 + t * 16 + row) * LDROW + kk);
#pragma unroll
                        for (int c = 0; c < NT; c++) {
                            acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[c][st][i], ah, acc[c][t], 0, 0, 0);
                            acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[c][st][i], al, acc[c][t], 0, 0, 0);
                        }
                    }
                }
            }
        }
        if (more) {
            w_issue(ch + 1);
            a_commit((ch + 1) & 1);
        }
        __syncthreads();
    }
    // epilogue: lane (m' = row, grp) holds D[n = 4*grp + r][m'] of each of its tiles
#pragma unroll
    for (int t = 0; t < MT; t++) {
        f32x4 v[NT];
#pragma unroll
        for (int c = 0; c < NT; c++) {
            v[c] = acc[c][t];
            if (PACKED) {
#pragma unroll
                for (int r = 0; r < 4; r++) v[c][r] += __shfl_xor(v[c][r], 8, 64); // hi half + lo half
            }
        }
        const int m = PACKED ? row : m0 + t * 16 + row;
        if ((PACKED && row >= 8) || m >= M) continue;
        if (MODE == GEMM_SWIGLU) {
#pragma unroll
            for (int j = 0; j < NT / 2; j++) {
                const size_t o = (size_t)m * N + n0 + (wave * (NT / 2) + j) * 16 + 4 * grp;
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const float g0 = v[2 * j][r];
                    const float y = g0 / (1.0f + expf(-g0)) * v[2 * j + 1][r];
                    const uint16_t hi = bf16_bits_rne(y);
                    Cact[o + r] = hi;
                    Cact[c_plane + o + r] = bf16_bits_rne(y - __uint_as_float((uint32_t)hi << 16));
                }
            }
        } else {
            float *Cs = C + (size_t)blockIdx.y * c_split_stride;
#pragma unroll
            for (int c = 0; c < NT; c++) {
                const size_t o = (size_t)m * N + n0 + (wave * NT + c) * 16 + 4 * grp;
                *(f32x4 *)(Cs + o) = v[c];
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
template <int NMAT, bool PACKED, int MT, int U, int NTW>
__global__ __launch_bounds__(256) void gemm_ksplit_kernel(const uint16_t *__restrict__ A, size_t a_plane, WeightSeg w,
                                                          int M, int N, int K, int steps_per_split,
                                                          float *__restrict__ C, size_t c_split_stride,
                                                          uint16_t *__restrict__ Cact, size_t c_plane)
{
    constexpr int WAVES = 4;
    constexpr int NW = NMAT * NTW; // weight tiles per wave and step
    __shared__ float red[WAVES][NW][MT][64][4];
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
        Ap[t] = A + ((PACKED && row >= 8) ? a_plane : 0) + (size_t)(a_live[t] ? m : 0) * K + grp * 8;
        Al[t] = Ap[t] + a_plane;
    }
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
                av[b][t][i] = a_live[t] ? *(const bf16x8 *)(Ap[t] + st * 128 + i * 32) : zero;
                if (!PACKED) al[b][t][i] = a_live[t] ? *(const bf16x8 *)(Al[t] + st * 128 + i * 32) : zero;
            }
#pragma unroll
        for (int c = 0; c < NW; c++)
#pragma unroll
            for (int i = 0; i < 4; i++)
                wv[b][c][i] = *(const bf16x8 *)(Wp[c % NMAT] + (size_t)(c / NMAT) * tile_elems + (size_t)st * 2048 + i * 512);
    };
#pragma unroll
    for (int u = 0; u < U; u++)
        if (s_begin + wave + u * WAVES < s_end) issue(s_begin + wave + u * WAVES, u);
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
            }
        }
    }
#pragma unroll
    for (int c = 0; c < NW; c++)
#pragma unroll
        for (int t = 0; t < MT; t++)
#pragma unroll
            for (int r = 0; r < 4; r++) red[wave][c][t][lane][r] = acc[c][t][r];
    __syncthreads();
    // tile element D[n = 4*(slot/16) + r][m' = slot%16] sits at red[.][c][t][slot][r]
    constexpr int ROWS = PACKED ? 8 : 16 * MT;
    for (int e = threadIdx.x; e < 16 * NTW * ROWS; e += 256) {
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
        }
        const size_t o = (size_t)m * N + n0 + j * 16 + nn;
        if (NMAT == 2) {
            const float y = v[0] / (1.0f + expf(-v[0])) * v[NMAT - 1];
            const uint16_t hi = bf16_bits_rne(y);
            Cact[o] = hi;
            Cact[c_plane + o] = bf16_bits_rne(y - __uint_as_float((uint32_t)hi << 16));
        } else {
            C[(size_t)blockIdx.y * c_split_stride + o] = v[0];
        }
    }
}

template <int MODE, int NT, int WAVES>
static void stream_launch(hipStream_t s, const uint16_t *a, size_t a_plane, WeightSeg w, int M, int N, int K, int ks,
                          float *C, size_t c_split_stride, uint16_t *ca, size_t c_plane)
{
    constexpr int COLS = (MODE == GEMM_SWIGLU ? NT / 2 : NT) * 16 * WAVES;
    int kps, ny;
    split_geometry(K, ks, &kps, &ny);
    const int ntiles = N / COLS;
    dim3 block(WAVES * 64);
    if (M <= 8)
        hipLaunchKernelGGL((gemm_stream_kernel<MODE, 16, 512, NT, WAVES>), dim3(ntiles, ny), block, 0, s, a, a_plane, w,
                           M, N, K, kps, 0, ntiles, C, c_split_stride, ca, c_plane);
    else if (M <= 16)
        hipLaunchKernelGGL((gemm_stream_kernel<MODE, 32, 256, NT, WAVES>), dim3(ntiles, ny), block, 0, s, a, a_plane, w,
                           M, N, K, kps, 0, ntiles, C, c_split_stride, ca, c_plane);
    else if (M <= 32)
        hipLaunchKernelGGL((gemm_stream_kernel<MODE, 64, 128, NT, WAVES>), dim3(ntiles, ny), block, 0, s, a, a_plane, w,
                           M, N, K, kps, 0, ntiles, C, c_split_stride, ca, c_plane);
    else {
        const int nmb = (M + 47) / 48;
        const int gx = ((ntiles + 7) / 8) * 8 * nmb;
        hipLaunchKernelGGL((gemm_stream_kernel<MODE, 96, 128, NT, WAVES>), dim3(gx, ny), block, 0, s, a, a_plane, w, M,
                           N, K, kps, nmb, ntiles, C, c_split_stride, ca, c_plane);
    }
}

int g_skinny_tune[3][2] = {{4, 0}, {4, 0}, {4, 0}}; // [mode] -> {waves per block, K splits (0 = automatic)}

// Number of K splits the launcher will use for this shape (the caller sizes and reduces the partials).
int gemm_skinny_splits(int mode, int M, int N, int K)
{
    if (mode == GEMM_SWIGLU || K < 128 || K % 128 != 0) return 1; // (the launcher rejects such K)
    int kps, ny;
    if (g_skinny_tune[mode][1] > 0) {
        split_geometry(K, g_skinny_tune[mode][1], &kps, &ny);
        return ny;
    }
    int blocks, target;
    if (M <= 16 && g_skinny_tune[mode][0] == 4) { // K-split kernel: 32 columns per block, each wave at least 2 steps
        blocks = N / 32;
        const int steps = K / 128;
        int ks = steps >= 16 ? 2 : 1; // measured: two half-length blocks per tile stream faster than one
        while (blocks * ks < 256 && ks < 8 && steps / (ks * 2) >= 4) ks *= 2;
        split_geometry(K, ks, &kps, &ny);
        return ny;
    }
    if (M <= 32) {
        blocks = N / (16 * g_skinny_tune[mode][0]);
        target = 768; // about three blocks per CU
    } else {
        blocks = (N / 128) * ((M + 47) / 48); // 2 waves x 4 tiles = 128 columns per block, 48-row blocks
        target = 384;                          // partial slabs cost M*N*4 bytes each here: split sparingly
    }
    int ks = 1;
    while (blocks * ks < target && ks < 8 && K / (ks * 2) >= 512) ks *= 2;
    split_geometry(K, ks, &kps, &ny);
    return ny;
}

// mode GEMM_STORE: C receives `splits` partial slabs [split][M][N] (split stride c_split_stride floats);
// mode GEMM_SWIGLU: Cact receives the bf16 hi/lo planes.  GEMM_RESID is expressed by the caller as a
// store into partial slabs followed by the fused add + norm kernel.
hipError_t launch_gemm_skinny_bf16(hipStream_t s, int mode, const void *A, size_t a_plane, WeightSeg w, int M, int N,
                                   int K, float *C, size_t c_split_stride, int splits, void *Cact, size_t c_plane)
{
    if (M < 1 || K % 128 != 0 || K < 128 || (mode != GEMM_STORE && mode != GEMM_SWIGLU)) return hipErrorNotSupported;
    if (!w.tiled) return hipErrorNotSupported; // these kernels read the 16 x 128 tile order only
    for (int i = 0; i < 3; i++)
        if (w.p[i] && ((uintptr_t)w.p[i] & 15)) return hipErrorNotSupported;
    if (((uintptr_t)A & 15) || (a_plane & 7) || (N & 3)) return hipErrorNotSupported;
    const uint16_t *a = (const uint16_t *)A;
    uint16_t *ca = (uint16_t *)Cact;
    const int waves = g_skinny_tune[mode][0];
    if (M > 32) { // row-blocked: 2 waves x 4 tiles per block
        if (mode == GEMM_SWIGLU) {
            if (N % 64 != 0) return hipErrorNotSupported;
            stream_launch<GEMM_SWIGLU, 4, 2>(s, a, a_plane, w, M, N, K, 1, C, 0, ca, c_plane);
        } else {
            if (N % 128 != 0 || w.n_per_seg % 128 != 0) return hipErrorNotSupported;
            stream_launch<GEMM_STORE, 4, 2>(s, a, a_plane, w, M, N, K, splits, C, c_split_stride, ca, c_plane);
        }
        return hipGetLastError();
    }
    if (mode == GEMM_SWIGLU && g_skinny_tune[GEMM_SWIGLU][1] == 0) { // default: K split inside the block
        if (N % 16 != 0) return hipErrorNotSupported;
        dim3 grid(N / 16), block(256);
#define SD_KSPLIT(NMAT, PACKED, MT, U, NTW, GRID, SPS)                                                              \
    hipLaunchKernelGGL((gemm_ksplit_kernel<NMAT, PACKED, MT, U, NTW>), GRID, dim3(256), 0, s, a, a_plane, w, M, N, K, \
                       SPS, C, c_split_stride, ca, c_plane)
        if (M <= 8) SD_KSPLIT(2, true, 1, 2, 1, grid, K / 128);
        else if (M <= 16) SD_KSPLIT(2, false, 1, 2, 1, grid, K / 128);
        else SD_KSPLIT(2, false, 2, 1, 1, grid, K / 128);
        return hipGetLastError();
    }
    if (mode == GEMM_STORE && waves == 4 && M <= 16 && N % 32 == 0 && w.n_per_seg % 32 == 0) {
        int kps, ny;
        split_geometry(K, splits, &kps, &ny);
        dim3 grid(N / 32, ny);
        if (M <= 8) SD_KSPLIT(1, true, 1, 2, 2, grid, kps / 128);
        else SD_KSPLIT(1, false, 1, 2, 2, grid, kps / 128);
        return hipGetLastError();
    }
    if (mode == GEMM_SWIGLU) {
        if (waves == 4 && N % 64 == 0) stream_launch<GEMM_SWIGLU, 2, 4>(s, a, a_plane, w, M, N, K, 1, C, 0, ca, c_plane);
        else if (waves == 8 && N % 128 == 0) stream_launch<GEMM_SWIGLU, 2, 8>(s, a, a_plane, w, M, N, K, 1, C, 0, ca, c_plane);
        else if (N % 32 == 0) stream_launch<GEMM_SWIGLU, 2, 2>(s, a, a_plane, w, M, N, K, 1, C, 0, ca, c_plane);
        else return hipErrorNotSupported;
        return hipGetLastError();
    }
    if (waves == 8 && N % 128 == 0 && w.n_per_seg % 128 == 0)
        stream_launch<GEMM_STORE, 1, 8>(s, a, a_plane, w, M, N, K, splits, C, c_split_stride, ca, c_plane);
    else if (N % 64 == 0 && w.n_per_seg % 64 == 0)
        stream_launch<GEMM_STORE, 1, 4>(s, a, a_plane, w, M, N, K, splits, C, c_split_stride, ca, c_plane);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}
