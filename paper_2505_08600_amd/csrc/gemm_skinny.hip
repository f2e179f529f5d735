// bf16 weight-streaming GEMM for few rows (M <= 32): C[M][N] = A[M][K] . W[N][K]^T.
//
// This is the verify forward at batch 1 (M = gamma+1) and every draft step: the
// work is reading each weight once from HBM, so the kernel is organised around
// the weight stream, and the matrix cores only keep the ALUs out of the way.
//
//  * a wave owns 16-column tiles of W: two of them (or, for SwiGLU, the gate and
//    the up tile of the same 16 columns) in the store / SwiGLU variants, one in the
//    residual variant, and walks K in steps of 128 elements; the waves of a block
//    interleave those steps (in-block split-K), so a block reads whole contiguous
//    kilobytes of every weight row per round;
//  * every lane loads 64 contiguous bytes of its weight row per step straight into
//    MFMA operand registers (v_mfma_f32_16x16x32_bf16: lane l supplies row l%16,
//    k-group l/16); the contraction index is permuted identically for both
//    operands, which a dot product does not care about;
//  * the activation operand comes from global memory (L2 hits), masked to the M
//    real rows; activations are two bf16 planes (hi + lo, ~16 mantissa bits), so
//    every weight fragment is multiplied twice - free while the kernel waits on HBM;
//  * the partial accumulators of the waves meet in LDS; the epilogue stores, adds
//    into the fp32 residual stream, or applies silu(gate)*up and rounds to bf16.
//    The sum order is fixed, so results are bit-reproducible run to run.
//
// Paper (arXiv 2505.08600): Section 1, Figure 1 (draft steps and the parallel
// verify pass whose linear layers these are); Section 3.1 (LLaMA blocks).
#include "sd_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define SK_KSTEP 128

// MT: 16-row tiles of A; WAVES: waves per block (in-block split-K); U: K steps in flight per wave
template <int MT, int MODE, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(const uint16_t *__restrict__ A, size_t a_plane,
                                                                 WeightSeg w, int M, int N, int K,
                                                                 float *__restrict__ C, uint16_t *__restrict__ Cact,
                                                                 size_t c_plane)
{
    constexpr bool DUAL = MODE != GEMM_RESID;
    constexpr int NT = DUAL ? 2 : 1;
    __shared__ float red[WAVES][NT][MT][64][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = lane & 15, grp = lane >> 4;
    int n0;
    const uint16_t *Wp[NT];
    if (MODE == GEMM_SWIGLU) {
        n0 = blockIdx.x * 16;
        Wp[0] = (const uint16_t *)w.p[0] + (size_t)(n0 + row) * K;
        Wp[NT - 1] = (const uint16_t *)w.p[1] + (size_t)(n0 + row) * K;
    } else {
        n0 = blockIdx.x * 16 * NT;
        int seg = n0 / w.n_per_seg;
        int nl = n0 - seg * w.n_per_seg;
        Wp[0] = (const uint16_t *)w.p[seg] + (size_t)(nl + row) * K;
        if (DUAL) Wp[NT - 1] = Wp[0] + (size_t)16 * K;
    }
    f32x4 acc[NT][MT];
#pragma unroll
    for (int c = 0; c < NT; c++)
#pragma unroll
        for (int t = 0; t < MT; t++) acc[c][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const int nsteps = K / SK_KSTEP;
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int s0 = wave * U; s0 < nsteps; s0 += WAVES * U) {
        bf16x8 wv[U][NT][4], av[U][MT][4], al[U][MT][4];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const bool live = s0 + u < nsteps;
            const int k = (live ? s0 + u : s0) * SK_KSTEP + grp * 32;
#pragma unroll
            for (int c = 0; c < NT; c++) {
                const bf16x8 *p = (const bf16x8 *)(Wp[c] + k);
#pragma unroll
                for (int i = 0; i < 4; i++) wv[u][c][i] = live ? p[i] : zero;
            }
#pragma unroll
            for (int t = 0; t < MT; t++) {
                const int m = t * 16 + row;
                const bf16x8 *pa = (const bf16x8 *)(A + (size_t)(m < M ? m : 0) * K + k);
                const bf16x8 *pl = (const bf16x8 *)(A + a_plane + (size_t)(m < M ? m : 0) * K + k);
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    av[u][t][i] = (live && m < M) ? pa[i] : zero;
                    al[u][t][i] = (live && m < M) ? pl[i] : zero;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++)
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int t = 0; t < MT; t++)
#pragma unroll
                    for (int c = 0; c < NT; c++) {
                        acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[u][c][i], av[u][t][i], acc[c][t], 0, 0, 0);
                        acc[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[u][c][i], al[u][t][i], acc[c][t], 0, 0, 0);
                    }
    }
#pragma unroll
    for (int c = 0; c < NT; c++)
#pragma unroll
        for (int t = 0; t < MT; t++)
#pragma unroll
            for (int r = 0; r < 4; r++) red[wave][c][t][lane][r] = acc[c][t][r];
    __syncthreads();
    // element (slot, r) of a tile is D[n = 4*(slot/16)+r][m = slot%16]; 256 of them per tile
    for (int e = threadIdx.x; e < 256; e += WAVES * 64) {
        const int slot = e & 63, r = e >> 6;
        const int nn = 4 * (slot >> 4) + r;
#pragma unroll
        for (int t = 0; t < MT; t++) {
            const int m = t * 16 + (slot & 15);
            float v[NT];
#pragma unroll
            for (int c = 0; c < NT; c++) {
                v[c] = 0.f;
#pragma unroll
                for (int wv2 = 0; wv2 < WAVES; wv2++) v[c] += red[wv2][c][t][slot][r];
            }
            if (m < M) {
                if (MODE == GEMM_SWIGLU) {
                    float g = v[0];
                    float y = g / (1.0f + expf(-g)) * v[NT - 1];
                    uint16_t hi = bf16_bits_rne(y);
                    Cact[(size_t)m * N + n0 + nn] = hi;
                    Cact[c_plane + (size_t)m * N + n0 + nn] = bf16_bits_rne(y - __uint_as_float((uint32_t)hi << 16));
                } else if (MODE == GEMM_STORE) {
                    C[(size_t)m * N + n0 + nn] = v[0];
                    C[(size_t)m * N + n0 + 16 + nn] = v[NT - 1];
                } else {
                    C[(size_t)m * N + n0 + nn] += v[0];
                }
            }
        }
    }
}

template <int MT>
static void skinny_dispatch(hipStream_t s, int mode, const void *A, size_t a_plane, WeightSeg w, int M, int N, int K,
                            float *C, void *Cact, size_t c_plane)
{
    const uint16_t *a = (const uint16_t *)A;
    uint16_t *ca = (uint16_t *)Cact;
    if (mode == GEMM_SWIGLU)
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, GEMM_SWIGLU, 4, 2>), dim3(N / 16), dim3(256), 0, s, a, a_plane, w,
                           M, N, K, C, ca, c_plane);
    else if (mode == GEMM_STORE)
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, GEMM_STORE, 4, 2>), dim3(N / 32), dim3(256), 0, s, a, a_plane, w, M,
                           N, K, C, ca, c_plane);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, GEMM_RESID, 8, 2>), dim3(N / 16), dim3(512), 0, s, a, a_plane, w, M,
                           N, K, C, ca, c_plane);
}

hipError_t launch_gemm_skinny_bf16(hipStream_t s, int mode, const void *A, size_t a_plane, WeightSeg w, int M, int N,
                                   int K, float *C, void *Cact, size_t c_plane)
{
    if (M < 1 || M > 32 || K % SK_KSTEP != 0) return hipErrorNotSupported;
    if (mode == GEMM_STORE) {
        if (N % 32 != 0 || w.n_per_seg % 32 != 0) return hipErrorNotSupported;
    } else if (N % 16 != 0) {
        return hipErrorNotSupported;
    }
    for (int i = 0; i < 3; i++)
        if (w.p[i] && ((uintptr_t)w.p[i] & 15)) return hipErrorNotSupported;
    if (((uintptr_t)A & 15) || (a_plane & 7)) return hipErrorNotSupported;
    if (M <= 16) skinny_dispatch<1>(s, mode, A, a_plane, w, M, N, K, C, Cact, c_plane);
    else skinny_dispatch<2>(s, mode, A, a_plane, w, M, N, K, C, Cact, c_plane);
    return hipGetLastError();
}
