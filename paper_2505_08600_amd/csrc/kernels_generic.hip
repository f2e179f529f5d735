// Reference-quality HIP kernels of the draft/verify path: they work for every
// supported shape in fp32 and bf16.  The fp32 (tiny) configuration runs on these
// alone; bf16 models use the MFMA kernels of the other files where their shape
// constraints hold and fall back here otherwise.
//
// Paper (arXiv 2505.08600): Section 1 / Figure 1 (draft rows, verify rows),
// Section 3.1 (LLaMA blocks; speculative-sampling verification, greedy limit).
#include "sd_internal.h"
#include <algorithm>

#define WAVE 64

// ---------------------------------------------------------------- block helpers
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}

// The one-block-per-row kernels (norms, samplers, the verify tail) spend their time waiting in block
// reductions, not computing.  These variants use the cross-lane data path of the vector ALU (DPP) instead
// of LDS shuffles, combine the 16 waves' partial results one entry per lane, and use barriers that wait
// for LDS traffic only, so that global stores issued before a reduction (the updated residual row, the q
// row a sampler has just written) drain behind it instead of stalling its first barrier.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ int row16_max(int v)
{
    v = max(v, dpp_i<0xB1>(v));
    v = max(v, dpp_i<0x4E>(v));
    v = max(v, dpp_i<0x141>(v));
    v = max(v, dpp_i<0x140>(v));
    return v;
}
// smallest value over the wave's 64 lanes (every lane gets it)
__device__ __forceinline__ int wave_min_i(int v)
{
    int m = row16_max(~v); // ~ reverses the order of ints
    m = max(max(__builtin_amdgcn_readlane(m, 0), __builtin_amdgcn_readlane(m, 16)),
            max(__builtin_amdgcn_readlane(m, 32), __builtin_amdgcn_readlane(m, 48)));
    return ~m;
}
__device__ __forceinline__ int wave_max_i(int v)
{
    const int m = row16_max(v);
    return max(max(__builtin_amdgcn_readlane(m, 0), __builtin_amdgcn_readlane(m, 16)),
               max(__builtin_amdgcn_readlane(m, 32), __builtin_amdgcn_readlane(m, 48)));
}
// Inverse-CDF placement inside one thread's four weights (indices i0 .. i0 + 3), the running sum continued from
// `cum`: the first index of positive weight whose inclusive sum exceeds the target, 0x7fffffff if there is none.
// Every thread of a scan evaluates it, whatever its starting sum, and the smallest index wins.  A thread's
// starting sum comes out of a parallel scan and is not bit-equal to its predecessor's sequentially added final
// sum, so a target within rounding of a thread boundary can be "not yet reached" at the end of one thread and
// "already passed" at the start of the next: then the next index of positive weight is the answer (and, because
// of the weight test, never an index the distribution gives no mass to).
__device__ __forceinline__ int first_over(float cum, const float4 f, float target, int i0)
{
    int k = 0x7fffffff;
    cum += f.x;
    if (f.x > 0.f && cum > target) k = i0;
    cum += f.y;
    if (k == 0x7fffffff && f.y > 0.f && cum > target) k = i0 + 1;
    cum += f.z;
    if (k == 0x7fffffff && f.z > 0.f && cum > target) k = i0 + 2;
    cum += f.w;
    if (k == 0x7fffffff && f.w > 0.f && cum > target) k = i0 + 3;
    return k;
}
__device__ __forceinline__ int last_positive(const float4 f, int i0)
{
    return f.w > 0.f ? i0 + 3 : f.z > 0.f ? i0 + 2 : f.y > 0.f ? i0 + 1 : f.x > 0.f ? i0 : -1;
}
// largest value, lowest index among equals
__device__ __forceinline__ void take_better(float &v, int &i, float ov, int oi)
{
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}
__device__ __forceinline__ void row16_argmax(float &v, int &i)
{
    take_better(v, i, dpp_f<0xB1>(v), dpp_i<0xB1>(i));
    take_better(v, i, dpp_f<0x4E>(v), dpp_i<0x4E>(i));
    take_better(v, i, dpp_f<0x141>(v), dpp_i<0x141>(i));
    take_better(v, i, dpp_f<0x140>(v), dpp_i<0x140>(i));
}
// Inclusive prefix sum over the 64 lanes: four shifted adds inside each row, then the totals of the rows before.
__device__ __forceinline__ float wave_incl_scan_dpp(float v, int lane)
{
    v += dpp_f<0x111>(v);
    v += dpp_f<0x112>(v);
    v += dpp_f<0x114>(v);
    v += dpp_f<0x118>(v);
    const float t0 = lane_f(v, 15), t1 = lane_f(v, 31), t2 = lane_f(v, 47);
    const int row = lane >> 4;
    const float off = row == 0 ? 0.f : row == 1 ? t0 : row == 2 ? t0 + t1 : (t0 + t1) + t2;
    return off + v;
}
// Sum over a block of exactly 16 waves; every thread gets the result.  red: 16 floats of LDS.
__device__ __forceinline__ float block_sum16(float v, float *red)
{
    const int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE;
    v = wave_sum_dpp(v);
    lds_barrier();
    if (l == 0) red[w] = v;
    lds_barrier();
    return row16_sum(red[l & 15]);
}


// Sum over the block; every thread gets the result.  red: >= 32 floats of LDS.
__device__ float block_sum(float v, float *red)
{
    int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE, nw = (blockDim.x + WAVE - 1) / WAVE;
    v = wave_sum(v);
    __syncthreads();
    if (l == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; i++) t += red[i];
    return t;
}
__device__ float block_max(float v, float *red)
{
    int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE, nw = (blockDim.x + WAVE - 1) / WAVE;
    v = wave_max(v);
    __syncthreads();
    if (l == 0) red[w] = v;
    __syncthreads();
    float t = red[0];
    for (int i = 1; i < nw; i++) t = fmaxf(t, red[i]);
    return t;
}

// Block-wide (value, index) argmax, ties to the lowest index.
__device__ void block_argmax(float &v, int &idx, float *redv, int *redi)
{
    int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE, nw = (blockDim.x + WAVE - 1) / WAVE;
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) {
        float ov = __shfl_xor(v, o, WAVE);
        int oi = __shfl_xor(idx, o, WAVE);
        if (ov > v || (ov == v && oi < idx)) {
            v = ov;
            idx = oi;
        }
    }
    __syncthreads();
    if (l == 0) {
        redv[w] = v;
        redi[w] = idx;
    }
    __syncthreads();
    v = redv[0];
    idx = redi[0];
    for (int i = 1; i < nw; i++)
        if (redv[i] > v || (redv[i] == v && redi[i] < idx)) {
            v = redv[i];
            idx = redi[i];
        }
}

// Exclusive prefix sum of one value per thread over the block.  scratch: >= 32 floats.
__device__ float block_excl_scan(float v, float *scratch)
{
    int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE, nw = (blockDim.x + WAVE - 1) / WAVE;
    float inc = v;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        float t = __shfl_up(inc, o, WAVE);
        if (l >= o) inc += t;
    }
    __syncthreads();
    if (l == WAVE - 1) scratch[w] = inc;
    __syncthreads();
    float base = 0.f;
    for (int i = 0; i < w && i < nw; i++) base += scratch[i];
    return base + inc - v;
}

// ---------------------------------------------------------------- row plan
// Builds the row list of one forward from the device-resident sequence state and
// advances the model's cache length.  One thread per selected sequence.
#define PLAN_THREADS 256
__global__ void plan_kernel(int mode, int R, int n_seq, const int32_t *seq_ids, CtxView cv, int slot, int upto_off,
                            const int32_t *cand, int gamma, int cand_idx, int vocab, PlanView pv)
{
    __shared__ int s_len[PLAN_THREADS]; // cache length after this forward, per sequence slot (single-block launches)
    if (threadIdx.x < PLAN_THREADS) s_len[threadIdx.x] = -1;
    __syncthreads();
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n_seq; j += gridDim.x * blockDim.x) {
        int b = seq_ids ? seq_ids[j] : j;
        if (b < 0 || b >= cv.B) { // refuse out-of-range ids: mark every row unused
            atomicOr(cv.status, 4);
            pv.seq_b[j] = 0;
            pv.seq_kv0[j] = 0;
            pv.seq_nq[j] = 0;
            if (gridDim.x > 1 || n_seq == 1) pv.seq_order[j] = j;
            else s_len[j] = 0;
            for (int r = 0; r < R; r++) {
                pv.row_tok[j * R + r] = 0;
                pv.row_pos[j * R + r] = 0;
                pv.row_b[j * R + r] = 0;
                pv.row_valid[j * R + r] = 0;
            }
            pv.lm_row[j] = j * R;
            continue;
        }
        int n = cv.ntok[b];
        int *kvp = cv.kvlen + (size_t)slot * cv.B + b;
        int kv = *kvp;
        int cap = cv.cap[b];
        int64_t off = cv.off[b];
        int nq = 0, kv0 = kv;
        if (mode == PLAN_CATCHUP) {
            int avail = (n - upto_off) - kv;
            nq = avail < 0 ? 0 : (avail > R ? R : avail);
            // a draft call (upto_off == 0) needs the pending token in its last row: a cache further behind
            // than R tokens would draw its candidates from another position - refuse and flag it
            if (upto_off == 0 && avail > R) {
                atomicOr(cv.status, 64);
                nq = 0;
            }
            // (a sequence whose candidate count is 0 still feeds its catch-up rows, so that its draft cache
            // stays within two tokens of the sequence; its sampler draws nothing)
        } else if (mode == PLAN_CAND) {
            nq = 1;
        } else { // PLAN_VERIFY: rows (pending token, candidates) at positions n-1 ..
            nq = seq_gamma(cv, b, gamma) + 1; // (= R unless the context carries per-sequence candidate counts)
            if (kv != n - 1) atomicOr(cv.status, 2);
            kv0 = n - 1;
        }
        if (n < 1) { // an empty sequence has no pending token
            atomicOr(cv.status, 2);
            nq = 0;
        }
        if (kv0 < 0) kv0 = 0;
        if (kv0 + nq > cap) { // never write beyond the sequence's cache rows
            atomicOr(cv.status, 1);
            nq = cap - kv0 > 0 ? cap - kv0 : 0;
            if (mode == PLAN_VERIFY) nq = 0;
        }
        for (int r = 0; r < R; r++) {
            int row = j * R + r;
            int valid = r < nq;
            int tok = 0;
            if (valid) {
                if (mode == PLAN_CATCHUP) tok = cv.tokens[off + kv0 + r];
                else if (mode == PLAN_CAND) tok = cand[j * gamma + cand_idx];
                else tok = r == 0 ? cv.tokens[off + n - 1] : cand[j * gamma + (r - 1)];
                if (tok < 0 || tok >= vocab) { // never index the embedding table out of range
                    atomicOr(cv.status, 16);
                    tok = 0;
                }
            }
            pv.row_tok[row] = tok;
            pv.row_pos[row] = kv0 + r;
            pv.row_b[row] = b;
            pv.row_valid[row] = valid;
        }
        pv.seq_b[j] = b;
        pv.seq_kv0[j] = kv0;
        pv.seq_nq[j] = nq;
        if (gridDim.x > 1 || n_seq == 1) pv.seq_order[j] = j;
        else s_len[j] = nq > 0 ? kv0 + nq : 0;
        if (mode == PLAN_VERIFY) {
            for (int r = 0; r < R; r++) pv.lm_row[j * R + r] = j * R + r;
        } else {
            pv.lm_row[j] = j * R + (nq > 0 ? nq - 1 : 0);
        }
        *kvp = kv0 + nq;
    }
    // Longest sequences first: attention blocks start in seq_order, so the blocks still running when the
    // grid drains are the short ones.  (A launch of several blocks wrote the identity order above.)
    if (gridDim.x == 1 && n_seq > 1) {
        __syncthreads();
        const int j = threadIdx.x;
        if (j < n_seq) {
            const int mine = s_len[j];
            int rank = 0;
            for (int i = 0; i < n_seq; i++) rank += (s_len[i] > mine) || (s_len[i] == mine && i < j);
            pv.seq_order[rank] = j;
        }
    }
}

// Prefill plan: every selected sequence gets G consecutive row groups of R rows (plan slots j*G .. j*G+G-1),
// group g holding the next pending tokens R*g .. R*g+R-1 of the sequence at cache positions kv + R*g ..;
// groups past the pending tokens stay empty.  Each group is a sequence slot of its own to the kernels that
// follow (its rows attend to everything before them, including the rows of the earlier groups, which the
// cache-append kernel has written by then).  One thread per selected sequence.
__global__ void plan_prefill_kernel(int R, int G, int n_seq, const int32_t *seq_ids, CtxView cv, int slot, int upto_off,
                                    int vocab, PlanView pv)
{
    // one block per sequence; its threads share out the (group, row) pairs
    const int j = blockIdx.x;
    int b = seq_ids ? seq_ids[j] : j;
    int total = 0, kv = 0;
    int64_t off = 0;
    int *kvp = nullptr;
    if (b < 0 || b >= cv.B) { // refuse out-of-range ids: every group stays empty
        if (threadIdx.x == 0) atomicOr(cv.status, 4);
        b = 0;
    } else {
        const int n = cv.ntok[b], cap = cv.cap[b];
        kvp = cv.kvlen + (size_t)slot * cv.B + b;
        kv = *kvp;
        off = cv.off[b];
        if (kv < 0) kv = 0;
        total = (n - upto_off) - kv;
        if (n < 1 && threadIdx.x == 0) atomicOr(cv.status, 2); // an empty sequence has nothing to feed
        if (total < 0 || n < 1) total = 0;
        if (kv + total > cap) { // never write beyond the sequence's cache rows
            if (threadIdx.x == 0) atomicOr(cv.status, 1);
            total = cap - kv > 0 ? cap - kv : 0;
        }
        if (total > R * G) total = R * G;
    }
    __syncthreads(); // every thread has read the cache length before thread 0 advances it
    for (int i = threadIdx.x; i < G * R; i += blockDim.x) {
        const int g = i / R, r = i % R;
        const int sl = j * G + g, kv0 = kv + g * R;
        const int nq = total - g * R < 0 ? 0 : (total - g * R > R ? R : total - g * R);
        const int row = sl * R + r, valid = r < nq;
        int tok = 0;
        if (valid) {
            tok = cv.tokens[off + kv0 + r];
            if (tok < 0 || tok >= vocab) { // never index the embedding table out of range
                atomicOr(cv.status, 16);
                tok = 0;
            }
        }
        pv.row_tok[row] = tok;
        pv.row_pos[row] = kv0 + r;
        pv.row_b[row] = b;
        pv.row_valid[row] = valid;
        if (r == 0) {
            pv.seq_b[sl] = b;
            pv.seq_kv0[sl] = kv0;
            pv.seq_nq[sl] = nq;
            pv.seq_order[sl] = sl;
        }
    }
    if (threadIdx.x == 0) {
        pv.lm_row[j] = total > 0 ? (j * G + (total - 1) / R) * R + (total - 1) % R : j * G * R;
        if (kvp) *kvp = kv + total;
    }
}

hipError_t launch_plan_prefill(hipStream_t s, int R, int G, int n_seq, const int32_t *seq_ids, CtxView cv, int slot,
                               int upto_off, int vocab, PlanView pv)
{
    hipLaunchKernelGGL(plan_prefill_kernel, dim3(n_seq), dim3(PLAN_THREADS), 0, s, R, G, n_seq, seq_ids, cv, slot, upto_off,
                       vocab, pv);
    return hipGetLastError();
}

hipError_t launch_plan(hipStream_t s, int mode, int R, int n_seq, const int32_t *seq_ids, CtxView cv, int slot,
                       int upto_off, const int32_t *cand, int gamma, int cand_idx, int vocab, PlanView pv)
{
    int threads = PLAN_THREADS, blocks = (n_seq + threads - 1) / threads;
    hipLaunchKernelGGL(plan_kernel, dim3(blocks), dim3(threads), 0, s, mode, R, n_seq, seq_ids, cv, slot, upto_off,
                       cand, gamma, cand_idx, vocab, pv);
    return hipGetLastError();
}

// ---------------------------------------------------------------- embedding gather
template <typename T>
__global__ void embed_kernel(const T *E, const int32_t *row_tok, int d, float *x)
{
    int r = blockIdx.x;
    const T *src = E + (size_t)row_tok[r] * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)r * d + i] = to_float(src[i]);
}

hipError_t launch_embed(hipStream_t s, int dtype, const void *E, const int32_t *row_tok, int M, int d, float *x)
{
    if (dtype == SD_BF16)
        hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(M), dim3(256), 0, s, (const bf16_t *)E, row_tok, d, x);
    else
        hipLaunchKernelGGL(embed_kernel<float>, dim3(M), dim3(256), 0, s, (const float *)E, row_tok, d, x);
    return hipGetLastError();
}

// ---------------------------------------------------------------- RMSNorm
// out[j] = T( x[src] * rsqrt(mean(x[src]^2) + eps) * g ), src = row_map ? row_map[j] : j.
template <typename T>
__global__ void rmsnorm_kernel(const float *x, const float *g, const int32_t *row_map, int d, float eps, T *out,
                               ActView av)
{
    __shared__ float red[32];
    int j = blockIdx.x;
    int src = row_map ? row_map[j] : j;
    const float *xr = x + (size_t)src * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) ss += xr[i] * xr[i];
    ss = block_sum(ss, red);
    float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += blockDim.x) store_act(out, act_index(av, j, i, d), av.plane, xr[i] * inv * g[i]);
}

hipError_t launch_rmsnorm(hipStream_t s, int dtype, const float *x, const float *g, const int32_t *row_map,
                          int n_rows, int d, float eps, void *out, ActView out_av)
{
    if (dtype == SD_BF16)
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3(n_rows), dim3(256), 0, s, x, g, row_map, d, eps,
                           (bf16_t *)out, out_av);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(n_rows), dim3(256), 0, s, x, g, row_map, d, eps,
                           (float *)out, out_av);
    return hipGetLastError();
}

// ---------------------------------------------------------------- generic GEMM  C = A . W^T
// One wave per output column n, 16 rows of A per block row; lanes stride over K.
template <typename T, int MODE>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T *A, ActView a_av, WeightSeg w, int M, int N,
                                                           int K, float *C, T *Cact, ActView c_av)
{
    int n = blockIdx.x * 4 + threadIdx.x / WAVE;
    int lane = threadIdx.x % WAVE;
    int m0 = blockIdx.y * 16;
    if (n >= N) return;
    const T *W0, *W1 = nullptr;
    int nl = n; // row inside its segment
    if (MODE == GEMM_SWIGLU) {
        W0 = (const T *)w.p[0];
        W1 = (const T *)w.p[1];
    } else {
        int seg = n / w.n_per_seg;
        nl = n - seg * w.n_per_seg;
        W0 = (const T *)w.p[seg];
    }
    float acc[16], acc2[16];
#pragma unroll
    for (int m = 0; m < 16; m++) acc[m] = acc2[m] = 0.f;
    int mcount = M - m0 < 16 ? M - m0 : 16;
    for (int k = lane; k < K; k += WAVE) {
        const size_t wi = weight_index(nl, k, K, w.tiled);
        float wv = to_float(W0[wi]);
        float wv2 = MODE == GEMM_SWIGLU ? to_float(W1[wi]) : 0.f;
#pragma unroll
        for (int m = 0; m < 16; m++) {
            if (m < mcount) {
                float a = load_act(A, act_index(a_av, m0 + m, k, K), a_av.plane);
                acc[m] += a * wv;
                if (MODE == GEMM_SWIGLU) acc2[m] += a * wv2;
            }
        }
    }
#pragma unroll
    for (int m = 0; m < 16; m++) {
        acc[m] = wave_sum(acc[m]);
        if (MODE == GEMM_SWIGLU) acc2[m] = wave_sum(acc2[m]);
    }
    if (lane == 0) {
        for (int m = 0; m < mcount; m++) {
            size_t o = (size_t)(m0 + m) * N + n;
            if (MODE == GEMM_STORE) C[o] = acc[m];
            else if (MODE == GEMM_RESID) C[o] += acc[m];
            else {
                float g = acc[m];
                store_act(Cact, act_index(c_av, m0 + m, n, N), c_av.plane, g / (1.0f + expf(-g)) * acc2[m]);
            }
        }
    }
}

// Row-major -> tiled weight order, one 16-byte piece per thread (destination-linear, so stores coalesce).
__global__ __launch_bounds__(256) void retile_bf16_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                          int N, int K)
{
    const size_t n_vec = (size_t)N * K / 8;
    for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < n_vec; v += (size_t)gridDim.x * 256) {
        const size_t step = v >> 8;            // 256 pieces per 16 x 128 step
        const int piece = (int)(v & 255);
        const int i = piece >> 6, g = (piece >> 4) & 3, r = piece & 15;
        const size_t steps_per_tile = (size_t)(K >> 7);
        const size_t n = (step / steps_per_tile) * 16 + r;
        const size_t k = (step % steps_per_tile) * 128 + i * 32 + g * 8;
        dst[v] = src[(n * K + k) / 8];
    }
}

hipError_t launch_retile_bf16(hipStream_t s, const void *src, void *dst, int N, int K)
{
    if (N % 16 != 0 || K % 128 != 0) return hipErrorInvalidValue;
    const size_t n_vec = (size_t)N * K / 8;
    const int blocks = (int)std::min<size_t>((n_vec + 255) / 256, 8192);
    hipLaunchKernelGGL(retile_bf16_kernel, dim3(blocks), dim3(256), 0, s, (const uint4 *)src, (uint4 *)dst, N, K);
    return hipGetLastError();
}

template <typename T>
static void gemm_generic_dispatch(hipStream_t s, int mode, const void *A, ActView a_av, WeightSeg w, int M, int N,
                                  int K, float *C, void *Cact, ActView c_av)
{
    dim3 grid((N + 3) / 4, (M + 15) / 16), block(256);
    if (mode == GEMM_STORE)
        hipLaunchKernelGGL((gemm_generic_kernel<T, GEMM_STORE>), grid, block, 0, s, (const T *)A, a_av, w, M, N, K,
                           C, (T *)Cact, c_av);
    else if (mode == GEMM_RESID)
        hipLaunchKernelGGL((gemm_generic_kernel<T, GEMM_RESID>), grid, block, 0, s, (const T *)A, a_av, w, M, N, K,
                           C, (T *)Cact, c_av);
    else
        hipLaunchKernelGGL((gemm_generic_kernel<T, GEMM_SWIGLU>), grid, block, 0, s, (const T *)A, a_av, w, M, N, K,
                           C, (T *)Cact, c_av);
}

hipError_t launch_gemm_generic(hipStream_t s, int dtype, int mode, const void *A, ActView a_av, WeightSeg w, int M,
                               int N, int K, float *C, void *Cact, ActView c_av)
{
    if (dtype == SD_BF16) gemm_generic_dispatch<bf16_t>(s, mode, A, a_av, w, M, N, K, C, Cact, c_av);
    else gemm_generic_dispatch<float>(s, mode, A, a_av, w, M, N, K, C, Cact, c_av);
    return hipGetLastError();
}

// ---------------------------------------------------------------- RoPE + KV append
// Embedding gather fused with the first layer's RMSNorm: x[r] = E[token_r]; out[r] = rmsnorm(x[r]) * g.
// Row r of one forward, by a whole block (red: 32 floats of LDS).  The element-wise form has the same
// element-to-thread assignment and reduction as rmsnorm_kernel (identical to the two separate launches); the
// vector form sums the squares in another order.
// bf16 rows whose width is a multiple of 8: 16-byte loads and stores, the row kept in registers between the two
// passes (a thread's 8 columns stay inside one 128-column step of the step-major order).
__device__ void embed_rmsnorm_row_vec(const bf16_t *E, int tok, int r, int d, float *x, const float *g, float eps,
                                      bf16_t *out, ActView av, float *red)
{
    constexpr int KEEP = 4; // 8-column pieces a thread holds (d <= 8 * KEEP * blockDim.x, else the rest is re-read)
    const uint4 *src = (const uint4 *)(E + (size_t)tok * d);
    float *xr = x + (size_t)r * d;
    const int npiece = d >> 3;
    float v[KEEP][8];
    float ss = 0.f;
    int it = 0;
    for (int p = threadIdx.x; p < npiece; p += blockDim.x, it++) {
        const uint4 w = src[p];
        const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
        float f[8];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            f[2 * e] = __uint_as_float(ws[e] << 16);
            f[2 * e + 1] = __uint_as_float(ws[e] & 0xffff0000u);
        }
        *(float4 *)(xr + 8 * p) = make_float4(f[0], f[1], f[2], f[3]);
        *(float4 *)(xr + 8 * p + 4) = make_float4(f[4], f[5], f[6], f[7]);
#pragma unroll
        for (int e = 0; e < 8; e++) {
            ss += f[e] * f[e];
            if (it < KEEP) v[it < KEEP ? it : 0][e] = f[e];
        }
    }
    ss = block_sum(ss, red); // (its barriers also make the x row visible to the re-reads below)
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    it = 0;
    for (int p = threadIdx.x; p < npiece; p += blockDim.x, it++) {
        float f[8];
        if (it < KEEP) {
#pragma unroll
            for (int e = 0; e < 8; e++) f[e] = v[it < KEEP ? it : 0][e];
        } else {
            const float4 a = *(const float4 *)(xr + 8 * p), b = *(const float4 *)(xr + 8 * p + 4);
            f[0] = a.x, f[1] = a.y, f[2] = a.z, f[3] = a.w, f[4] = b.x, f[5] = b.y, f[6] = b.z, f[7] = b.w;
        }
        const float4 g0 = *(const float4 *)(g + 8 * p), g1 = *(const float4 *)(g + 8 * p + 4);
        const size_t o = act_index(av, r, 8 * p, d);
        store_act4(out, o, av.plane, f[0] * inv * g0.x, f[1] * inv * g0.y, f[2] * inv * g0.z, f[3] * inv * g0.w);
        store_act4(out, o + 4, av.plane, f[4] * inv * g1.x, f[5] * inv * g1.y, f[6] * inv * g1.z, f[7] * inv * g1.w);
    }
}
template <typename T>
__device__ void embed_rmsnorm_row(const T *E, int tok, int r, int d, float *x, const float *g, float eps, T *out,
                                  ActView av, float *red)
{
    if constexpr (sizeof(T) == 2) {
        if ((d & 7) == 0) { // (uniform)
            embed_rmsnorm_row_vec(E, tok, r, d, x, g, eps, out, av, red);
            return;
        }
    }
    const T *src = E + (size_t)tok * d;
    float *xr = x + (size_t)r * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        const float v = to_float(src[i]);
        xr[i] = v;
        ss += v * v;
    }
    ss = block_sum(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += blockDim.x)
        store_act(out, act_index(av, r, i, d), av.plane, to_float(src[i]) * inv * g[i]);
}

template <typename T>
__global__ __launch_bounds__(256) void embed_rmsnorm_kernel(const T *E, const int32_t *row_tok, int d, float *x,
                                                            const float *g, float eps, T *out, ActView av)
{
    __shared__ float red[32];
    embed_rmsnorm_row(E, row_tok[blockIdx.x], blockIdx.x, d, x, g, eps, out, av, red);
}

hipError_t launch_embed_rmsnorm(hipStream_t s, int dtype, const void *E, const int32_t *row_tok, int M, int d, float *x,
                                const float *g, float eps, void *out, ActView out_av)
{
    if (dtype == SD_BF16)
        hipLaunchKernelGGL(embed_rmsnorm_kernel<bf16_t>, dim3(M), dim3(256), 0, s, (const bf16_t *)E, row_tok, d, x, g,
                           eps, (bf16_t *)out, out_av);
    else
        hipLaunchKernelGGL(embed_rmsnorm_kernel<float>, dim3(M), dim3(256), 0, s, (const float *)E, row_tok, d, x, g,
                           eps, (float *)out, out_av);
    return hipGetLastError();
}

// qkv: fp32 [M][3*HD] (q | k | v).  Rotates q and k of every valid row at its
// position (rotate-half pairing), writes q to qbuf and k, v into the cache in
// place: K in 32-token tiles in MFMA operand order (kt_offset), V in 32-token transposed tiles (vt_offset).
// Residual update fused with the next RMSNorm: x[src] += sum of the split-K slabs of the
// preceding GEMM (added in slab order), then out[j] = rmsnorm(x[src]) * g.  One block of 1024
// threads per row; the loads of all slabs of an element are independent and go out together.
#define ROPE_MAX_SLABS 8
// (MAX_SLABS: 8 covers the K splits of the GEMMs; 16 the per-head slabs an attention kernel that applies the
// output projection itself leaves for a small model)
template <typename T, int ADDNORM_MAX_SLABS>
__global__ __launch_bounds__(1024) void add_rmsnorm_kernel(float *x, const float *part, int n_slabs, size_t slab_stride,
                                                           const float *g, const int32_t *row_map, int d, float eps,
                                                           T *out, ActView av)
{
    __shared__ float red[16];
    int j = blockIdx.x;
    int src = row_map ? row_map[j] : j;
    float *xr = x + (size_t)src * d;
    const float *pr = part + (size_t)src * d;
    float ss = 0.f;
    const int nvec = d / 4; // d is a multiple of 4 (checked at load)
    constexpr int KEEP = 2; // vectors of the row a thread keeps in registers (d <= 8192)
    float4 keep[KEEP], gain[KEEP];
    int it = 0;
    for (int v = threadIdx.x; v < nvec; v += blockDim.x, it++) {
        float4 a = *(const float4 *)(xr + 4 * v);
        float4 p[ADDNORM_MAX_SLABS];
#pragma unroll
        for (int s = 0; s < ADDNORM_MAX_SLABS; s++)
            if (s < n_slabs) p[s] = *(const float4 *)(pr + (size_t)s * slab_stride + 4 * v);
        // the gains are needed only after the reduction; loaded there they would add a memory round trip
        if (it < KEEP) gain[it] = *(const float4 *)(g + 4 * v);
#pragma unroll
        for (int s = 0; s < ADDNORM_MAX_SLABS; s++)
            if (s < n_slabs) {
                a.x += p[s].x;
                a.y += p[s].y;
                a.z += p[s].z;
                a.w += p[s].w;
            }
        *(float4 *)(xr + 4 * v) = a;
        if (it < KEEP) keep[it] = a;
        ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
    }
    ss = block_sum16(ss, red); // 1024 threads; does not wait for the residual stores above
    if (nvec > KEEP * (int)blockDim.x) __syncthreads(); // wider rows are read back below: let the stores land
    float inv = 1.0f / sqrtf(ss / (float)d + eps);
    it = 0;
    for (int v = threadIdx.x; v < nvec; v += blockDim.x, it++) {
        const float4 a = it < KEEP ? keep[it] : *(const float4 *)(xr + 4 * v);
        const float4 gg = it < KEEP ? gain[it] : *(const float4 *)(g + 4 * v);
        const size_t o = act_index(av, j, 4 * v, d); // 4 consecutive columns stay inside one K step
        store_act4(out, o, av.plane, a.x * inv * gg.x, a.y * inv * gg.y, a.z * inv * gg.z, a.w * inv * gg.w);
    }
}

hipError_t launch_add_rmsnorm(hipStream_t s, int dtype, float *x, const float *part, int n_slabs, size_t slab_stride,
                              const float *g, const int32_t *row_map, int n_rows, int d, float eps, void *out,
                              ActView out_av)
{
    if (n_slabs > 16 || (d & 3)) return hipErrorInvalidValue;
    if (dtype == SD_BF16 && n_slabs > 8)
        hipLaunchKernelGGL((add_rmsnorm_kernel<bf16_t, 16>), dim3(n_rows), dim3(1024), 0, s, x, part, n_slabs, slab_stride,
                           g, row_map, d, eps, (bf16_t *)out, out_av);
    else if (dtype == SD_BF16)
        hipLaunchKernelGGL((add_rmsnorm_kernel<bf16_t, 8>), dim3(n_rows), dim3(1024), 0, s, x, part, n_slabs, slab_stride,
                           g, row_map, d, eps, (bf16_t *)out, out_av);
    else if (n_slabs > 8)
        return hipErrorInvalidValue;
    else
        hipLaunchKernelGGL((add_rmsnorm_kernel<float, 8>), dim3(n_rows), dim3(1024), 0, s, x, part, n_slabs, slab_stride,
                           g, row_map, d, eps, (float *)out, out_av);
    return hipGetLastError();
}

// ---------------------------------------------------------------- low-rank adapters
// One block per row.  The row (hi + lo summed) goes to LDS; the 4 waves share the n_proj * rank dot
// products with the A factors; every thread then produces outputs n = tid, tid + 256, ...
#define LORA_MAX_RANK 16
#define LORA_MAX_K 8192
struct LoraPtrs {
    const float *a[3], *b[3];
};
template <typename T>
__global__ __launch_bounds__(256) void lora_delta_kernel(const T *X, ActView x_av, int K, int N, int n_proj, PlanView pv,
                                                         const int32_t *adapter, int n_adapters, int rank, float scale,
                                                         LoraPtrs lp, float *out, int accumulate)
{
    __shared__ __attribute__((aligned(16))) float sx[LORA_MAX_K];
    __shared__ float st[3][LORA_MAX_RANK];
    const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int a = pv.row_valid[r] ? adapter[pv.row_b[r]] : -1;
    if (a >= n_adapters) a = -1;
    float *orow = out + (size_t)r * n_proj * N;
    if (a < 0) {
        if (!accumulate)
            for (int n = threadIdx.x; n < n_proj * N; n += 256) orow[n] = 0.f;
        return;
    }
    for (int k = threadIdx.x; k < K; k += 256) sx[k] = load_act(X, act_index(x_av, r, k, K), x_av.plane);
    __syncthreads();
    // wave w takes the dot products pj = w, w + 4, ...: six at a time, so that their loads are in flight together
    constexpr int PJ = 6;
    for (int pj0 = wave; pj0 < n_proj * rank; pj0 += 4 * PJ) {
        const float *arow[PJ];
        float acc[PJ];
#pragma unroll
        for (int u = 0; u < PJ; u++) {
            const int pj = pj0 + 4 * u;
            const int p = pj < n_proj * rank ? pj / rank : 0, j = pj % rank;
            arow[u] = pj < n_proj * rank && lp.a[p] ? lp.a[p] + ((size_t)a * rank + j) * K : nullptr;
            acc[u] = 0.f;
        }
#pragma unroll 2
        for (int k = 4 * lane; k < K; k += 256) { // 16 bytes per lane and load (K is a multiple of 4)
            const float4 xv = *(const float4 *)&sx[k];
#pragma unroll
            for (int u = 0; u < PJ; u++)
                if (arow[u]) {
                    const float4 av = *(const float4 *)(arow[u] + k);
                    acc[u] += av.x * xv.x + av.y * xv.y + av.z * xv.z + av.w * xv.w;
                }
        }
#pragma unroll
        for (int u = 0; u < PJ; u++) {
            float v = acc[u];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            const int pj = pj0 + 4 * u;
            if (lane == 0 && pj < n_proj * rank) st[pj / rank][pj % rank] = v;
        }
    }
    __syncthreads();
    // outputs n = tid, tid + 256, ...: four at a time (independent loads of the B rows)
    const int n_out = n_proj * N;
    for (int n0 = threadIdx.x; n0 < n_out; n0 += 4 * 256) {
        float acc[4], old[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int n = n0 + 256 * u;
            acc[u] = 0.f;
            old[u] = 0.f;
            if (n < n_out) {
                const int p = n / N, nn = n % N;
                if (accumulate) old[u] = orow[n];
                if (lp.a[p] && lp.b[p]) {
                    const float *brow = lp.b[p] + ((size_t)a * N + nn) * rank;
                    float bv[LORA_MAX_RANK]; // all loads of the row go out before the first is used
#pragma unroll
                    for (int j = 0; j < LORA_MAX_RANK; j++) bv[j] = j < rank ? brow[j] : 0.f;
#pragma unroll
                    for (int j = 0; j < LORA_MAX_RANK; j++)
                        if (j < rank) acc[u] += bv[j] * st[p][j];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int n = n0 + 256 * u;
            if (n < n_out) orow[n] = old[u] + scale * acc[u];
        }
    }
}

hipError_t launch_lora_delta(hipStream_t s, int dtype, const void *X, ActView x_av, int M, int K, int N, int n_proj,
                             PlanView pv, const int32_t *adapter, int n_adapters, int rank, float scale,
                             const float *const *A, const float *const *B, float *out, int accumulate)
{
    if (M < 1 || K < 4 || (K & 3) || K > LORA_MAX_K || n_proj < 1 || n_proj > 3 || rank < 1 || rank > LORA_MAX_RANK || !adapter)
        return hipErrorInvalidValue;
    LoraPtrs lp;
    for (int p = 0; p < 3; p++) lp.a[p] = p < n_proj ? A[p] : nullptr, lp.b[p] = p < n_proj ? B[p] : nullptr;
    if (dtype == SD_BF16)
        hipLaunchKernelGGL(lora_delta_kernel<bf16_t>, dim3(M), dim3(256), 0, s, (const bf16_t *)X, x_av, K, N, n_proj, pv,
                           adapter, n_adapters, rank, scale, lp, out, accumulate);
    else
        hipLaunchKernelGGL(lora_delta_kernel<float>, dim3(M), dim3(256), 0, s, (const float *)X, x_av, K, N, n_proj, pv,
                           adapter, n_adapters, rank, scale, lp, out, accumulate);
    return hipGetLastError();
}

template <typename T>
__global__ void rope_append_kernel(const float *qkv, int n_slabs, size_t slab_stride, PlanView pv, CtxView cv, int H,
                                   int hd, const float2 *rope,
                                   int max_pos, T *qbuf, ActView q_av, T *Kl, T *Vtl, int64_t total_cap)
{
    int r = blockIdx.x;
    int HD = H * hd, half = hd / 2;
    int valid = pv.row_valid[r];
    int pos = pv.row_pos[r];
    if (pos >= max_pos) {
        if (threadIdx.x == 0 && valid) atomicOr(cv.status, 8);
        valid = 0;
    }
    const float *row = qkv + (size_t)r * 3 * HD;
    int64_t off = cv.off[pv.row_b[r]];
    for (int i = threadIdx.x; i < H * half; i += blockDim.x) {
        int h = i / half, e = i % half;
        if (!valid) {
            store_act(qbuf, act_index(q_av, r, h * hd + e, HD), q_av.plane, 0.f);
            store_act(qbuf, act_index(q_av, r, h * hd + e + half, HD), q_av.plane, 0.f);
            continue;
        }
        float2 cs = rope[(size_t)pos * half + e];
        float q0 = 0.f, q1 = 0.f, k0 = 0.f, k1 = 0.f, v0 = 0.f, v1 = 0.f;
        float ld[ROPE_MAX_SLABS][6];
#pragma unroll
        for (int sl = 0; sl < ROPE_MAX_SLABS; sl++) // split-K slabs of the QKV GEMM: all loads go out first
            if (sl < n_slabs) {
                const float *rs = row + (size_t)sl * slab_stride;
                ld[sl][0] = rs[h * hd + e];
                ld[sl][1] = rs[h * hd + e + half];
                ld[sl][2] = rs[HD + h * hd + e];
                ld[sl][3] = rs[HD + h * hd + e + half];
                ld[sl][4] = rs[2 * HD + h * hd + e];
                ld[sl][5] = rs[2 * HD + h * hd + e + half];
            }
#pragma unroll
        for (int sl = 0; sl < ROPE_MAX_SLABS; sl++) // ... and are added in slab order
            if (sl < n_slabs) {
                q0 += ld[sl][0];
                q1 += ld[sl][1];
                k0 += ld[sl][2];
                k1 += ld[sl][3];
                v0 += ld[sl][4];
                v1 += ld[sl][5];
            }
        store_act(qbuf, act_index(q_av, r, h * hd + e, HD), q_av.plane, q0 * cs.x - q1 * cs.y);
        store_act(qbuf, act_index(q_av, r, h * hd + e + half, HD), q_av.plane, q1 * cs.x + q0 * cs.y);
        T *kh = Kl + (size_t)h * total_cap * hd;
        kh[kt_offset(hd, off + pos, e)] = from_float<T>(k0 * cs.x - k1 * cs.y);
        kh[kt_offset(hd, off + pos, e + half)] = from_float<T>(k1 * cs.x + k0 * cs.y);
        T *vh = Vtl + (size_t)h * hd * total_cap;
        vh[vt_offset(hd, off + pos, e)] = from_float<T>(v0);
        vh[vt_offset(hd, off + pos, e + half)] = from_float<T>(v1);
    }
}

// The same step for bf16 models with head width 64 or 128, one block per (head, group of up to 16 rows whose
// positions follow each other).  The row-per-block kernel above writes every cache element with a 2-byte store
// of its own - V elements of consecutive dimensions lie 64 bytes apart in the transposed tiles - and takes 27 us
// for 576 rows of the 7B shape.  Here a thread owns 8 consecutive dimensions of both rotary halves of one row:
// float4 loads of the slabs (added in slab order, like above: same bits), 16-byte stores of the two q planes and
// of the K pieces (8 consecutive dimensions of a token are one piece of the operand-order tile); the V values go
// through LDS so that a thread can write the 16 tokens of one dimension as 32 contiguous bytes when the group is
// full and starts at a multiple of 16 (every prefill group of a fresh prompt), and token by token otherwise.
template <int HD>
__global__ __launch_bounds__(HD) void rope_append_group_kernel(const float *__restrict__ qkv, int n_slabs, size_t slab_stride,
                                                               PlanView pv, CtxView cv, int R, int H,
                                                               const float2 *__restrict__ rope, int max_pos,
                                                               uint16_t *__restrict__ qbuf, ActView q_av,
                                                               uint16_t *__restrict__ Kl, uint16_t *__restrict__ Vtl,
                                                               int64_t total_cap)
{
    constexpr int HALF = HD / 2, GPR = HALF / 8; // 8-dimension groups per rotary half
    __shared__ __attribute__((aligned(16))) uint16_t sV[16][HD + 8];
    __shared__ int s_pos[16];
    const int h = blockIdx.x, j = blockIdx.y;
    const int i = threadIdx.x / GPR, g = threadIdx.x % GPR; // row of the group, dimension group
    const int HDm = H * HD;
    const int r = j * R + min(i, R - 1);
    int valid = i < R && pv.row_valid[r];
    const int pos = pv.row_pos[r];
    if (valid && pos >= max_pos) {
        if (g == 0 && h == 0) atomicOr(cv.status, 8);
        valid = 0;
    }
    const int64_t off = cv.off[pv.row_b[r]];
    const int d0 = 8 * g, d1 = HALF + 8 * g;
    float q[16], k[16], v[16]; // [0..7]: dimensions d0.., [8..15]: d1..
#pragma unroll
    for (int e = 0; e < 16; e++) q[e] = k[e] = v[e] = 0.f;
    if (valid) {
        const float *base = qkv + (size_t)r * 3 * HDm + h * HD;
        for (int sl = 0; sl < n_slabs; sl++) { // split-K slabs of the QKV GEMM, added in slab order
            const float *rs = base + (size_t)sl * slab_stride;
            float4 ld[12];
#pragma unroll
            for (int m = 0; m < 3; m++) {
                ld[4 * m + 0] = *(const float4 *)(rs + m * HDm + d0);
                ld[4 * m + 1] = *(const float4 *)(rs + m * HDm + d0 + 4);
                ld[4 * m + 2] = *(const float4 *)(rs + m * HDm + d1);
                ld[4 * m + 3] = *(const float4 *)(rs + m * HDm + d1 + 4);
            }
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const float4 a = ld[c], b = ld[4 + c], w = ld[8 + c];
                q[4 * c + 0] += a.x, q[4 * c + 1] += a.y, q[4 * c + 2] += a.z, q[4 * c + 3] += a.w;
                k[4 * c + 0] += b.x, k[4 * c + 1] += b.y, k[4 * c + 2] += b.z, k[4 * c + 3] += b.w;
                v[4 * c + 0] += w.x, v[4 * c + 1] += w.y, v[4 * c + 2] += w.z, v[4 * c + 3] += w.w;
            }
        }
        const float2 *cs = rope + (size_t)pos * HALF + d0;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const float2 c = cs[e];
            const float qa = q[e] * c.x - q[8 + e] * c.y, qb = q[8 + e] * c.x + q[e] * c.y;
            const float ka = k[e] * c.x - k[8 + e] * c.y, kb = k[8 + e] * c.x + k[e] * c.y;
            q[e] = qa, q[8 + e] = qb, k[e] = ka, k[8 + e] = kb;
        }
    }
    if (i < R) { // q planes (zeros for rows without a token), 8 consecutive columns inside one K step
#pragma unroll
        for (int hf = 0; hf < 2; hf++) {
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; e++) bf16x2_split(q[8 * hf + 2 * e], q[8 * hf + 2 * e + 1], hi[e], lo[e]);
            const size_t o = act_index(q_av, r, h * HD + (hf ? d1 : d0), HDm);
            *(uint4 *)(qbuf + o) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            *(uint4 *)(qbuf + o + q_av.plane) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
    }
    if (valid) {
        uint16_t *kh = Kl + (size_t)h * total_cap * HD;
#pragma unroll
        for (int hf = 0; hf < 2; hf++) {
            uint32_t p[4];
#pragma unroll
            for (int e = 0; e < 4; e++) p[e] = bf16x2_bits_rne(k[8 * hf + 2 * e], k[8 * hf + 2 * e + 1]);
            *(uint4 *)(kh + kt_offset(HD, off + pos, hf ? d1 : d0)) = make_uint4(p[0], p[1], p[2], p[3]);
#pragma unroll
            for (int e = 0; e < 4; e++) p[e] = bf16x2_bits_rne(v[8 * hf + 2 * e], v[8 * hf + 2 * e + 1]);
            *(uint4 *)&sV[i][hf ? d1 : d0] = make_uint4(p[0], p[1], p[2], p[3]);
        }
    }
    if (g == 0) s_pos[i] = valid ? pos : -1;
    __syncthreads();
    // V: thread d writes dimension d of the group's tokens
    const int d = threadIdx.x;
    uint16_t *vh = Vtl + (size_t)h * HD * total_cap;
    const int p0 = s_pos[0];
    bool run16 = p0 >= 0 && (p0 & 15) == 0;
#pragma unroll
    for (int t = 1; t < 16; t++) run16 = run16 && s_pos[t] == p0 + t;
    const int64_t off0 = cv.off[pv.row_b[j * R]]; // (one sequence per group)
    if (run16) {
        uint32_t p[8];
#pragma unroll
        for (int t = 0; t < 8; t++) p[t] = (uint32_t)sV[2 * t][d] | ((uint32_t)sV[2 * t + 1][d] << 16);
        uint16_t *dst = vh + vt_offset(HD, off0 + p0, d); // 16 tokens inside one 32-token tile: 32 contiguous bytes
        *(uint4 *)dst = make_uint4(p[0], p[1], p[2], p[3]);
        *(uint4 *)(dst + 8) = make_uint4(p[4], p[5], p[6], p[7]);
    } else {
        for (int t = 0; t < 16; t++)
            if (s_pos[t] >= 0) vh[vt_offset(HD, off0 + s_pos[t], d)] = sV[t][d];
    }
}

int g_rope_group = 1; // option "rope_group": 0 keeps the row-per-block kernel for bf16 models too
hipError_t launch_rope_append(hipStream_t s, int dtype, const float *qkv, int n_slabs, size_t slab_stride, PlanView pv,
                              CtxView cv, int M, int R, int H, int hd, const float2 *rope, int max_pos, void *qbuf,
                              ActView q_av, void *Kl, void *Vtl, int64_t total_cap)
{
    if (n_slabs > ROPE_MAX_SLABS) return hipErrorInvalidValue;
    if (dtype == SD_BF16 && g_rope_group && R >= 1 && R <= 16 && M % R == 0 && (hd == 64 || hd == 128) && H <= 65535 &&
        M / R <= 65535 && (q_av.plane & 7) == 0 && ((uintptr_t)qbuf & 15) == 0 && ((uintptr_t)Kl & 15) == 0 &&
        ((uintptr_t)Vtl & 15) == 0 && ((uintptr_t)qkv & 15) == 0 && (slab_stride & 3) == 0 && total_cap % 64 == 0) {
        if (hd == 128)
            hipLaunchKernelGGL(rope_append_group_kernel<128>, dim3(H, M / R), dim3(128), 0, s, qkv, n_slabs, slab_stride, pv,
                               cv, R, H, rope, max_pos, (uint16_t *)qbuf, q_av, (uint16_t *)Kl, (uint16_t *)Vtl, total_cap);
        else
            hipLaunchKernelGGL(rope_append_group_kernel<64>, dim3(H, M / R), dim3(64), 0, s, qkv, n_slabs, slab_stride, pv, cv,
                               R, H, rope, max_pos, (uint16_t *)qbuf, q_av, (uint16_t *)Kl, (uint16_t *)Vtl, total_cap);
        return hipGetLastError();
    }
    if (dtype == SD_BF16)
        hipLaunchKernelGGL(rope_append_kernel<bf16_t>, dim3(M), dim3(1024), 0, s, qkv, n_slabs, slab_stride, pv, cv, H,
                           hd, rope, max_pos, (bf16_t *)qbuf, q_av, (bf16_t *)Kl, (bf16_t *)Vtl, total_cap);
    else
        hipLaunchKernelGGL(rope_append_kernel<float>, dim3(M), dim3(1024), 0, s, qkv, n_slabs, slab_stride, pv, cv, H,
                           hd, rope, max_pos, (float *)qbuf, q_av, (float *)Kl, (float *)Vtl, total_cap);
    return hipGetLastError();
}

// ---------------------------------------------------------------- generic attention
// One block per (row slot i, head, selected sequence): query row i sees cache rows
// [0, kv0 + i].  Scores live in dynamic LDS (lds_len floats: the largest sequence capacity).
template <typename T>
__global__ __launch_bounds__(256) void attn_generic_kernel(const T *qbuf, ActView q_av, const T *Kl, const T *Vtl,
                                                           PlanView pv, CtxView cv, int R, int H, int hd,
                                                           int64_t total_cap, int lds_len, T *obuf, ActView o_av)
{
    extern __shared__ float sc[]; // [lds_len] scores, then [256] partials, [hd] q, [32] red
    float *part = sc + lds_len;
    float *qs = part + 256;
    float *red = qs + hd;
    int i = blockIdx.x, h = blockIdx.y, j = blockIdx.z;
    int r = j * R + i;
    int HD = H * hd;
    if (i >= pv.seq_nq[j]) {
        for (int d = threadIdx.x; d < hd; d += blockDim.x) store_act(obuf, act_index(o_av, r, h * hd + d, HD), o_av.plane, 0.f);
        return;
    }
    int Lk = pv.seq_kv0[j] + i + 1;
    if (Lk > lds_len) { // the launch was sized for fewer rows than the cache holds: flag it, do not read on
        if (threadIdx.x == 0) atomicOr(cv.status, 32);
        Lk = lds_len;
    }
    int64_t off = cv.off[pv.seq_b[j]];
    const T *Kh = Kl + (size_t)h * total_cap * hd;
    const T *Vh = Vtl + (size_t)h * hd * total_cap;
    for (int d = threadIdx.x; d < hd; d += blockDim.x) qs[d] = load_act(qbuf, act_index(q_av, r, h * hd + d, HD), q_av.plane);
    __syncthreads();
    float scale = 1.0f / sqrtf((float)hd);
    float mx = -3.0e38f;
    for (int t = threadIdx.x; t < Lk; t += blockDim.x) {
        float dot = 0.f;
        for (int d = 0; d < hd; d++) dot += qs[d] * to_float(Kh[kt_offset(hd, off + t, d)]);
        dot *= scale;
        sc[t] = dot;
        mx = fmaxf(mx, dot);
    }
    mx = block_max(mx, red);
    float z = 0.f;
    for (int t = threadIdx.x; t < Lk; t += blockDim.x) {
        float e = expf(sc[t] - mx);
        sc[t] = e;
        z += e;
    }
    z = block_sum(z, red);
    __syncthreads();
    int G = blockDim.x / hd; // hd is 64 or 128, blockDim 256
    int d = threadIdx.x % hd, g = threadIdx.x / hd;
    float acc = 0.f;
    for (int t = g; t < Lk; t += G) acc += sc[t] * to_float(Vh[vt_offset(hd, off + t, d)]);
    part[threadIdx.x] = acc;
    __syncthreads();
    if (g == 0) {
        for (int gg = 1; gg < G; gg++) acc += part[gg * hd + d];
        store_act(obuf, act_index(o_av, r, h * hd + d, HD), o_av.plane, acc / z);
    }
}

hipError_t launch_attn_generic(hipStream_t s, int dtype, const void *qbuf, ActView q_av, const void *Kl,
                               const void *Vtl, PlanView pv, CtxView cv, int R, int n_seq, int H, int hd,
                               int64_t total_cap, int len_upper, void *obuf, ActView o_av)
{
    size_t lds = ((size_t)len_upper + 256 + hd + 32) * sizeof(float);
    if (lds > 160 * 1024) return hipErrorNotSupported;
    if (lds > 64 * 1024) { // beyond the default limit: ask for the larger LDS allocation this part has
        hipError_t ea = dtype == SD_BF16
                            ? hipFuncSetAttribute((const void *)attn_generic_kernel<bf16_t>,
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                            : hipFuncSetAttribute((const void *)attn_generic_kernel<float>,
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (ea != hipSuccess) return hipErrorNotSupported;
    }
    dim3 grid(R, H, n_seq), block(256);
    if (dtype == SD_BF16)
        hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, grid, block, lds, s, (const bf16_t *)qbuf, q_av,
                           (const bf16_t *)Kl, (const bf16_t *)Vtl, pv, cv, R, H, hd, total_cap, len_upper,
                           (bf16_t *)obuf, o_av);
    else
        hipLaunchKernelGGL(attn_generic_kernel<float>, grid, block, lds, s, (const float *)qbuf, q_av,
                           (const float *)Kl, (const float *)Vtl, pv, cv, R, H, hd, total_cap, len_upper,
                           (float *)obuf, o_av);
    return hipGetLastError();
}

// ---------------------------------------------------------------- inverse-CDF pick
// Chooses the smallest index k with sum_{x<=k} w(x) > u * sum_x w(x) for weights
// produced on the fly by wfun(v) -> float4 of elements 4v..4v+3 (zero beyond V).
// All threads of a 1024-thread block must call it; the result is returned to all.
// The sums are added in parallel (segment totals, then a scan inside the segment that holds u * Z), so where
// rounding makes them disagree the answer is the nearest index of positive weight: see first_over; if no
// running sum of the chosen segment exceeds the target, the segment's last index of positive weight; if
// u * Z is not below Z at all, the row's last one.
struct PickScratch {
    float seg[64];
    float red[32];
    float base;
    float target;
    int seg_idx;
    int pick;
    int last_pos;
    int seg_last; // last index of positive weight inside the segment that holds the target
};

template <typename F>
__device__ int block_pick_cdf(F wfun, int V, float u, PickScratch *ps, float *total_out)
{
    const int T = blockDim.x;
    int nvec = (V + 3) / 4;
    int nseg = (nvec + T - 1) / T;
    if (threadIdx.x == 0) {
        ps->pick = 0x7fffffff;
        ps->last_pos = 0;
        ps->seg_last = -1;
    }
    __syncthreads();
    int lastp = -1;
    for (int it = 0; it < nseg; it++) {
        int v = it * T + threadIdx.x;
        float4 f = v < nvec ? wfun(v) : make_float4(0.f, 0.f, 0.f, 0.f);
        if (f.x > 0.f) lastp = 4 * v;
        if (f.y > 0.f) lastp = 4 * v + 1;
        if (f.z > 0.f) lastp = 4 * v + 2;
        if (f.w > 0.f) lastp = 4 * v + 3;
        float loc = ((f.x + f.y) + f.z) + f.w;
        float ssum = block_sum(loc, ps->red);
        if (threadIdx.x == 0) ps->seg[it] = ssum;
    }
    if (lastp >= 0) atomicMax(&ps->last_pos, lastp);
    __syncthreads();
    if (threadIdx.x == 0) {
        float Z = 0.f;
        for (int it = 0; it < nseg; it++) Z += ps->seg[it];
        float target = u * Z;
        float cum = 0.f;
        int found = -1;
        for (int it = 0; it < nseg; it++) {
            if (cum + ps->seg[it] > target) {
                found = it;
                break;
            }
            cum += ps->seg[it];
        }
        ps->seg_idx = found;
        ps->base = cum;
        ps->target = target;
        if (total_out) *total_out = Z;
    }
    __syncthreads();
    int it = ps->seg_idx;
    if (it >= 0) {
        int v = it * T + threadIdx.x;
        float4 f = v < nvec ? wfun(v) : make_float4(0.f, 0.f, 0.f, 0.f);
        float loc = ((f.x + f.y) + f.z) + f.w;
        float pre = block_excl_scan(loc, ps->red);
        int k = first_over(ps->base + pre, f, ps->target, 4 * v);
        if (k >= V) k = 0x7fffffff;
        k = wave_min_i(k);
        const int ls = wave_max_i(last_positive(f, 4 * v));
        if (threadIdx.x % WAVE == 0) {
            if (k != 0x7fffffff) atomicMin(&ps->pick, k);
            if (ls >= 0) atomicMax(&ps->seg_last, ls);
        }
    }
    __syncthreads();
    int pick = ps->pick;
    // rounding left every running sum of the chosen segment at or below the target: its last index of positive
    // weight; no segment chosen (u * Z not below Z): the last one of the row
    if (pick == 0x7fffffff) pick = it >= 0 && ps->seg_last >= 0 ? min(ps->seg_last, V - 1) : ps->last_pos;
    __syncthreads();
    return pick;
}

__device__ __forceinline__ float4 load4_guard(const float *row, int v, int V, float fill)
{
    if (4 * v + 3 < V) return *(const float4 *)(row + 4 * v);
    float4 f = make_float4(fill, fill, fill, fill);
    if (4 * v < V) f.x = row[4 * v];
    if (4 * v + 1 < V) f.y = row[4 * v + 1];
    if (4 * v + 2 < V) f.z = row[4 * v + 2];
    return f;
}

// max and lowest-index argmax of one fp32 row (block-wide)
__device__ void row_max_argmax(const float *row, int V, float *redv, int *redi, float &mx, int &am)
{
    float bv = -3.0e38f;
    int bi = 0x7fffffff;
    int nvec = (V + 3) / 4;
    for (int v = threadIdx.x; v < nvec; v += blockDim.x) {
        float4 f = load4_guard(row, v, V, -3.0e38f);
        if (f.x > bv) { bv = f.x; bi = 4 * v; }
        if (f.y > bv) { bv = f.y; bi = 4 * v + 1; }
        if (f.z > bv) { bv = f.z; bi = 4 * v + 2; }
        if (f.w > bv) { bv = f.w; bi = 4 * v + 3; }
    }
    block_argmax(bv, bi, redv, redi);
    mx = bv;
    am = bi;
}

// sum_x exp((row[x] - mx) * invT) (block-wide)
__device__ float row_sumexp(const float *row, int V, float mx, float invT, float *red)
{
    float z = 0.f;
    int nvec = (V + 3) / 4;
    for (int v = threadIdx.x; v < nvec; v += blockDim.x) {
        float4 f = load4_guard(row, v, V, -3.0e38f);
        z += expf((f.x - mx) * invT);
        if (4 * v + 1 < V) z += expf((f.y - mx) * invT);
        if (4 * v + 2 < V) z += expf((f.z - mx) * invT);
        if (4 * v + 3 < V) z += expf((f.w - mx) * invT);
    }
    return block_sum(z, red);
}

// ---------------------------------------------------------------- register-resident vocabulary rows
// For V <= 32768 a 1024-thread block holds a whole fp32 row in registers: thread t keeps the float4s
// number it*1024 + t, it < ROW_NSEG - the same element-to-thread assignment as the strided loops of the
// general kernels above; the block-wide sums are added as trees here, so the two paths agree to rounding
// (and exactly in the maximum and the arg max).  One pass over memory per row and a handful of barriers
// instead of one block reduction per 4096 elements.
#define ROW_NSEG 8
#define ROW_THREADS 1024
struct RowRegs {
    float4 f[ROW_NSEG];
};
struct FastScratch {
    float wsum[ROW_THREADS / WAVE][ROW_NSEG];
    float red[32];
    int redi[32];
    int pick;
    int seg_last; // last index of positive weight inside the segment that holds the target
};
static_assert(ROW_THREADS / WAVE == 16, "the cross-wave steps below read one LDS entry per lane of a 16-lane row");

// Block-wide arg max / sum for ROW_THREADS threads; every thread gets the result.
__device__ void block_argmax_rows(float &v, int &idx, FastScratch *fs)
{
    const int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE;
    row16_argmax(v, idx);
    float bv = lane_f(v, 0);
    int bi = __builtin_amdgcn_readlane(idx, 0);
    take_better(bv, bi, lane_f(v, 16), __builtin_amdgcn_readlane(idx, 16));
    take_better(bv, bi, lane_f(v, 32), __builtin_amdgcn_readlane(idx, 32));
    take_better(bv, bi, lane_f(v, 48), __builtin_amdgcn_readlane(idx, 48));
    lds_barrier();
    if (l == 0) {
        fs->red[w] = bv;
        fs->redi[w] = bi;
    }
    lds_barrier();
    v = fs->red[l & 15];
    idx = fs->redi[l & 15];
    row16_argmax(v, idx);
}
__device__ float block_sum_rows(float v, FastScratch *fs) { return block_sum16(v, fs->red); }

__device__ __forceinline__ void row_load(const float *row, int V, float fill, RowRegs &r)
{
    const int nvec = (V + 3) / 4;
#pragma unroll
    for (int it = 0; it < ROW_NSEG; it++) {
        const int v = it * ROW_THREADS + threadIdx.x;
        r.f[it] = v < nvec ? load4_guard(row, v, V, fill) : make_float4(fill, fill, fill, fill);
    }
}

// max, lowest-index argmax and (T > 0) z = sum of e(x) = exp((x - max) / T) of the row in r (filled with
// -3e38 past V).  For T > 0 the row is replaced by e(x) (exactly 0 past V), so that the probabilities
// e(x) / z need no second exponential.
__device__ void row_stats_regs(RowRegs &r, float invT, FastScratch *fs, float &mx, int &am, float &z)
{
    float bv = -3.0e38f;
    int bi = 0x7fffffff;
#pragma unroll
    for (int it = 0; it < ROW_NSEG; it++) {
        const int v = it * ROW_THREADS + threadIdx.x;
        const float4 f = r.f[it];
        if (f.x > bv) { bv = f.x; bi = 4 * v; }
        if (f.y > bv) { bv = f.y; bi = 4 * v + 1; }
        if (f.z > bv) { bv = f.z; bi = 4 * v + 2; }
        if (f.w > bv) { bv = f.w; bi = 4 * v + 3; }
    }
    block_argmax_rows(bv, bi, fs);
    mx = bv;
    am = bi;
    z = 1.f;
    if (invT > 0.f) {
        float zl = 0.f;
#pragma unroll
        for (int it = 0; it < ROW_NSEG; it++) {
            float4 f = r.f[it];
            f.x = expf((f.x - mx) * invT);
            f.y = expf((f.y - mx) * invT);
            f.z = expf((f.z - mx) * invT);
            f.w = expf((f.w - mx) * invT);
            zl += f.x;
            zl += f.y;
            zl += f.z;
            zl += f.w;
            r.f[it] = f;
        }
        z = block_sum_rows(zl, fs);
    }
}

// Inverse-CDF pick (same rule as block_pick_cdf) over weights held in registers.
__device__ int pick_regs(const RowRegs &w, int V, float u, FastScratch *fs, float *total_out)
{
    // Index order is (segment it, thread t, component c).  Segment totals are the waves' totals added as a
    // tree; every thread works out the total Z, the segment holding u * Z and the sum before it for itself
    // (no single-thread phase), then one block-wide scan of that segment's float4 sums places the element.
    const int lane = threadIdx.x % WAVE, wv = threadIdx.x / WAVE;
    int lastp = -1;
    float loc[ROW_NSEG];
#pragma unroll
    for (int it = 0; it < ROW_NSEG; it++) {
        const int v = it * ROW_THREADS + threadIdx.x;
        const float4 f = w.f[it];
        if (f.x > 0.f) lastp = 4 * v;
        if (f.y > 0.f) lastp = 4 * v + 1;
        if (f.z > 0.f) lastp = 4 * v + 2;
        if (f.w > 0.f) lastp = 4 * v + 3;
        loc[it] = wave_sum_dpp(((f.x + f.y) + f.z) + f.w);
    }
    lastp = row16_max(lastp);
    lastp = max(max(__builtin_amdgcn_readlane(lastp, 0), __builtin_amdgcn_readlane(lastp, 16)),
                max(__builtin_amdgcn_readlane(lastp, 32), __builtin_amdgcn_readlane(lastp, 48)));
    lds_barrier(); // the scratch may still be in use by a previous call
    if (lane == 0) {
#pragma unroll
        for (int it = 0; it < ROW_NSEG; it++) fs->wsum[wv][it] = loc[it];
        fs->redi[wv] = lastp;
    }
    if (threadIdx.x == 0) {
        fs->pick = 0x7fffffff;
        fs->seg_last = -1;
    }
    lds_barrier();
    const int nseg = ((V + 3) / 4 + ROW_THREADS - 1) / ROW_THREADS;
    float seg[ROW_NSEG];
#pragma unroll
    for (int it = 0; it < ROW_NSEG; it++) seg[it] = row16_sum(fs->wsum[lane & 15][it]);
    const int lp = max(row16_max(fs->redi[lane & 15]), 0); // last index with a positive weight (0 if there is none)
    float Z = 0.f;
#pragma unroll
    for (int it = 0; it < ROW_NSEG; it++)
        if (it < nseg) Z += seg[it];
    const float target = u * Z;
    float base = 0.f;
    int sit = -1;
#pragma unroll
    for (int it = 0; it < ROW_NSEG; it++)
        if (it < nseg && sit < 0) {
            if (base + seg[it] > target) sit = it;
            else base += seg[it];
        }
    if (total_out) *total_out = Z;
    if (sit >= 0) { // uniform over the block
        float4 f = w.f[0];
#pragma unroll
        for (int it = 1; it < ROW_NSEG; it++)
            if (it == sit) f = w.f[it];
        const int v = sit * ROW_THREADS + threadIdx.x;
        const float l4 = ((f.x + f.y) + f.z) + f.w;
        const float inc = wave_incl_scan_dpp(l4, lane);
        if (lane == WAVE - 1) fs->red[wv] = inc; // red was last read before the barrier above
        lds_barrier();
        const float before = row16_sum((lane & 15) < wv ? fs->red[lane & 15] : 0.f);
        int k = first_over(base + (before + inc - l4), f, target, 4 * v);
        if (k >= V) k = 0x7fffffff;
        k = wave_min_i(k);
        const int ls = wave_max_i(last_positive(f, 4 * v));
        if (lane == 0) {
            if (k != 0x7fffffff) atomicMin(&fs->pick, k);
            if (ls >= 0) atomicMax(&fs->seg_last, ls);
        }
    }
    lds_barrier();
    int pick = fs->pick;
    // rounding left every running sum of the chosen segment at or below the target: its last index of positive
    // weight; no segment chosen (u * Z not below Z): the last one of the row
    if (pick == 0x7fffffff) pick = sit >= 0 && fs->seg_last >= 0 ? min(fs->seg_last, V - 1) : lp;
    lds_barrier();
    return pick;
}

// e(x) -> probabilities e(x) * (1 / z), in place
__device__ __forceinline__ void row_scale(RowRegs &r, float invZ)
{
#pragma unroll
    for (int it = 0; it < ROW_NSEG; it++) {
        r.f[it].x *= invZ;
        r.f[it].y *= invZ;
        r.f[it].z *= invZ;
        r.f[it].w *= invZ;
    }
}

// The single-row plan (PLAN_CAND, R = 1) of sequence slot j for the forward that feeds `tok`: the same entries,
// checks and cache-length update as plan_kernel makes for that mode, written by the sampler block that has
// just drawn the token.  seq_order keeps the order the catch-up plan of this draft call left (every
// sequence grows by one row, so the ranking by length does not change).  One thread calls this.
__device__ int plan_next_cand(const NextPlan &np, int j, int tok)
{
    const PlanView &pv = np.pv;
    const CtxView &cv = np.cv;
    const int b = np.seq_ids ? np.seq_ids[j] : j;
    if (b < 0 || b >= cv.B) { // refuse out-of-range ids: the row stays unused
        atomicOr(cv.status, 4);
        pv.seq_b[j] = 0;
        pv.seq_kv0[j] = 0;
        pv.seq_nq[j] = 0;
        pv.row_tok[j] = 0;
        pv.row_pos[j] = 0;
        pv.row_b[j] = 0;
        pv.row_valid[j] = 0;
        pv.lm_row[j] = j;
        return 0;
    }
    const int n = cv.ntok[b];
    int *kvp = cv.kvlen + (size_t)np.slot * cv.B + b;
    int kv0 = *kvp, nq = 1;
    const int cap = cv.cap[b];
    if (np.next_idx >= seq_gamma(cv, b, np.gamma)) nq = 0; // the sequence has drawn all its candidates
    if (n < 1) { // an empty sequence has no pending token
        atomicOr(cv.status, 2);
        nq = 0;
    }
    if (kv0 < 0) kv0 = 0;
    if (kv0 + nq > cap) { // never write beyond the sequence's cache rows
        atomicOr(cv.status, 1);
        nq = cap - kv0 > 0 ? cap - kv0 : 0;
    }
    if (nq > 0 && (tok < 0 || tok >= np.vocab)) { // never index the embedding table out of range
        atomicOr(cv.status, 16);
        tok = 0;
    }
    pv.row_tok[j] = nq > 0 ? tok : 0;
    pv.row_pos[j] = kv0;
    pv.row_b[j] = b;
    pv.row_valid[j] = nq > 0;
    pv.seq_b[j] = b;
    pv.seq_kv0[j] = kv0;
    pv.seq_nq[j] = nq;
    pv.lm_row[j] = j;
    *kvp = kv0 + nq;
    return nq > 0 ? tok : 0; // (= row_tok[j]: what the planned forward embeds)
}

// Does sequence slot j draw candidate idx in this draft call?  With per-sequence candidate counts a sequence that
// has drawn all of its own sits the remaining forwards out: its rows are unused, nothing of it is written (the
// sampler that drew its last candidate has already left its plan entry empty).
__device__ __forceinline__ bool draft_seq_active(const NextPlan &np, int j, int gamma, int idx)
{
    if (!np.cv.gam) return true;
    const int b = np.seq_ids ? np.seq_ids[j] : j;
    if (b < 0 || b >= np.cv.B) return true; // (the plan has flagged it; behave as without counts)
    return idx < seq_gamma(np.cv, b, gamma);
}

__global__ __launch_bounds__(ROW_THREADS) void draft_sample_fast_kernel(const float *logits, int V, float T,
                                                                         const float *u, int gamma, int idx,
                                                                         int32_t *cand, float *q, NextPlan next)
{
    __shared__ FastScratch fs;
    const int j = blockIdx.x;
    if (!draft_seq_active(next, j, gamma, idx)) { // (uniform over the block) nothing to draw: keep its plan entry empty
        if (threadIdx.x == 0 && next.enabled) plan_next_cand(next, j, 0);
        return;
    }
    RowRegs r;
    row_load(logits + (size_t)j * V, V, -3.0e38f, r);
    float mx, z;
    int am;
    row_stats_regs(r, T > 0.f ? 1.0f / T : 0.f, &fs, mx, am, z);
    if (T == 0.f) {
        if (threadIdx.x == 0) {
            cand[j * gamma + idx] = am;
            if (next.enabled) plan_next_cand(next, j, am);
        }
        return;
    }
    row_scale(r, 1.0f / z);
    float *qrow = q + ((size_t)j * gamma + idx) * V;
    const int nvec = (V + 3) / 4;
#pragma unroll
    for (int it = 0; it < ROW_NSEG; it++) {
        const int v = it * ROW_THREADS + threadIdx.x;
        const float4 p = r.f[it];
        if (4 * v + 3 < V) *(float4 *)(qrow + 4 * v) = p;
        else if (v < nvec) {
            if (4 * v < V) qrow[4 * v] = p.x;
            if (4 * v + 1 < V) qrow[4 * v + 1] = p.y;
            if (4 * v + 2 < V) qrow[4 * v + 2] = p.z;
        }
    }
    const int pick = pick_regs(r, V, u[j * gamma + idx], &fs, nullptr);
    if (threadIdx.x == 0) {
        cand[j * gamma + idx] = pick;
        if (next.enabled) plan_next_cand(next, j, pick);
    }
}

// ---- samplers that start from the LM head's per-block softmax partials (LmStats: 32 columns per entry)
// A row's vocabulary is cut into slices of DS_SLICE columns, one 256-thread block each.  Every block reads all
// the row's partials (a few KB) and derives from them, in the same order and therefore to the same bits as
// every other block of the row: the row maximum, the mass of every slice (one wave-wide sum of the slice's 64
// entries), the normaliser Z (the slice masses added in order) and the slice in which the running sum first
// exceeds u * Z.  It then writes its own slice of q = exp((x - max) / T) / Z, and the one block that owns the
// slice holding u * Z places the candidate inside it with a block-wide scan (same rule as block_pick_cdf:
// first index whose inclusive sum exceeds the target, else the last index of positive weight).  No block waits
// for another.  The owner also lays out the next single-row forward and, if asked, runs its first step
// (embedding row + first norm).
#define DS_SLICE 2048
#define DS_MAX_SLICES 32
struct SplitScratch {
    float red[32];
    float wmax[4];
    float slice[DS_MAX_SLICES];
    float wtot[2][4];
    int pick, lastp, tok;
};

__device__ void next_forward_first_step(const NextPlan &next, int j, int tok, SplitScratch *ss)
{
    // (all threads of the block) thread 0 plans; then the block gathers and norms the row
    if (threadIdx.x == 0) ss->tok = next.enabled ? plan_next_cand(next, j, tok) : 0;
    if (!next.enabled || !next.embed) return;
    __syncthreads();
    embed_rmsnorm_row((const bf16_t *)next.E, ss->tok, j, next.d, next.x, next.g, next.eps, (bf16_t *)next.out, next.av,
                      ss->red);
}

__global__ __launch_bounds__(256) void draft_sample_split_kernel(const float *logits, const float *stats, int nb, int V,
                                                                  float T, const float *u, int gamma, int idx,
                                                                  int32_t *cand, float *q, NextPlan next)
{
    __shared__ SplitScratch ss;
    const int j = blockIdx.y, k = blockIdx.x, n_slices = gridDim.x;
    const int lane = threadIdx.x % WAVE, wv = threadIdx.x / WAVE;
    if (!draft_seq_active(next, j, gamma, idx)) { // (uniform over the block) nothing to draw: keep its plan entry empty
        if (k == 0) next_forward_first_step(next, j, 0, &ss);
        return;
    }
    const float invT = 1.0f / T;
    const float *st = stats + (size_t)j * nb * 3;
    // this block's slice of the logits row: requested first, needed only once the maximum and Z are known
    const float *row = logits + (size_t)j * V;
    float4 e[2];
#pragma unroll
    for (int it = 0; it < 2; it++) {
        const int v = k * (DS_SLICE / 4) + it * 256 + threadIdx.x; // (V is a multiple of 32: whole float4s only)
        e[it] = 4 * v < V ? *(const float4 *)(row + 4 * v) : make_float4(-3.0e38f, -3.0e38f, -3.0e38f, -3.0e38f);
    }
    // wave w holds the entries of slices w, w + 4, ...: lane l entry 64 * slice + l
    float em[DS_MAX_SLICES / 4], es[DS_MAX_SLICES / 4];
    float mx = -3.0e38f;
#pragma unroll
    for (int i = 0; i < DS_MAX_SLICES / 4; i++) {
        const int b = (4 * i + wv) * 64 + lane;
        const bool in = 4 * i + wv < n_slices && b < nb;
        em[i] = in ? st[3 * b] : -3.0e38f;
        es[i] = in ? st[3 * b + 1] : 0.f;
        mx = fmaxf(mx, em[i]);
    }
    mx = wave_max(mx);
    if (lane == 0) ss.wmax[wv] = mx;
    if (threadIdx.x == 0) {
        ss.pick = 0x7fffffff;
        ss.lastp = -1;
    }
    __syncthreads();
    mx = fmaxf(fmaxf(ss.wmax[0], ss.wmax[1]), fmaxf(ss.wmax[2], ss.wmax[3]));
#pragma unroll
    for (int i = 0; i < DS_MAX_SLICES / 4; i++) {
        const float mass = wave_sum_dpp(es[i] * expf((em[i] - mx) * invT)); // (entries past the row: 0 * 0)
        if (lane == 0 && 4 * i + wv < n_slices) ss.slice[4 * i + wv] = mass;
    }
    __syncthreads();
    float Z = 0.f, base = 0.f;
    for (int s = 0; s < n_slices; s++) {
        if (s == k) base = Z;
        Z += ss.slice[s];
    }
    const float target = u[j * gamma + idx] * Z;
    int owner = -1, last_pos = 0;
    {
        float cum = 0.f;
        for (int s = 0; s < n_slices; s++) {
            const float m = ss.slice[s];
            cum += m;
            if (m > 0.f) last_pos = s;
            if (owner < 0 && cum > target) owner = s;
        }
        if (owner < 0) owner = last_pos;
    }
    // this block's slice of q
    const float invZ = 1.0f / Z;
    float *qrow = q + ((size_t)j * gamma + idx) * V;
#pragma unroll
    for (int it = 0; it < 2; it++) {
        const int v = k * (DS_SLICE / 4) + it * 256 + threadIdx.x;
        if (4 * v < V) {
            float4 f = e[it];
            f.x = expf((f.x - mx) * invT);
            f.y = expf((f.y - mx) * invT);
            f.z = expf((f.z - mx) * invT);
            f.w = expf((f.w - mx) * invT);
            e[it] = f;
            *(float4 *)(qrow + 4 * v) = make_float4(f.x * invZ, f.y * invZ, f.z * invZ, f.w * invZ);
        } else {
            e[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    if (k != owner) return; // (uniform over the block)
    // place the target inside the slice: index order is (it, thread, component)
    float l4[2], inc[2];
    int lastp = -1;
#pragma unroll
    for (int it = 0; it < 2; it++) {
        const int v = k * (DS_SLICE / 4) + it * 256 + threadIdx.x;
        const float4 f = e[it];
        if (f.x > 0.f) lastp = 4 * v;
        if (f.y > 0.f) lastp = 4 * v + 1;
        if (f.z > 0.f) lastp = 4 * v + 2;
        if (f.w > 0.f) lastp = 4 * v + 3;
        l4[it] = ((f.x + f.y) + f.z) + f.w;
        inc[it] = wave_incl_scan_dpp(l4[it], lane);
        if (lane == WAVE - 1) ss.wtot[it][wv] = inc[it];
    }
    if (lastp >= 0) atomicMax(&ss.lastp, lastp);
    __syncthreads();
    float seg_before = base;
#pragma unroll
    for (int it = 0; it < 2; it++) {
        float before = seg_before;
        for (int w = 0; w < 4; w++) {
            if (w < wv) before += ss.wtot[it][w];
            seg_before += ss.wtot[it][w];
        }
        const int v = k * (DS_SLICE / 4) + it * 256 + threadIdx.x;
        const float4 f = e[it];
        int pk = first_over(before + (inc[it] - l4[it]), f, target, 4 * v);
        if (pk >= V) pk = 0x7fffffff;
        pk = wave_min_i(pk);
        if (lane == 0 && pk != 0x7fffffff) atomicMin(&ss.pick, pk);
    }
    __syncthreads();
    int pick = ss.pick;
    if (pick == 0x7fffffff) pick = max(ss.lastp, 0);
    if (threadIdx.x == 0) cand[j * gamma + idx] = pick;
    next_forward_first_step(next, j, pick, &ss);
}

// Greedy candidate from the partials: the largest block maximum, lowest column among equals.
__global__ __launch_bounds__(256) void draft_argmax_split_kernel(const float *stats, int nb, int gamma, int idx,
                                                                  int32_t *cand, NextPlan next)
{
    __shared__ SplitScratch ss;
    __shared__ int redi[32];
    const int j = blockIdx.x;
    if (!draft_seq_active(next, j, gamma, idx)) {
        next_forward_first_step(next, j, 0, &ss);
        return;
    }
    const float *st = stats + (size_t)j * nb * 3;
    float bv = -3.0e38f;
    int bi = 0x7fffffff;
    for (int b = threadIdx.x; b < nb; b += 256) take_better(bv, bi, st[3 * b], __float_as_int(st[3 * b + 2]));
    block_argmax(bv, bi, ss.red, redi);
    if (threadIdx.x == 0) cand[j * gamma + idx] = bi;
    __syncthreads(); // (block_argmax read ss.red last)
    next_forward_first_step(next, j, bi, &ss);
}

// ---------------------------------------------------------------- draft: softmax + sample
// One block per sequence.  T > 0: q = softmax(logits / T) is written in full and
// the candidate drawn by inverse CDF; T == 0: candidate = argmax.
__global__ __launch_bounds__(1024) void draft_sample_kernel(const float *logits, int V, float T, const float *u,
                                                            int gamma, int idx, int32_t *cand, float *q, NextPlan next)
{
    __shared__ PickScratch ps;
    __shared__ float redv[32];
    __shared__ int redi[32];
    int j = blockIdx.x;
    if (!draft_seq_active(next, j, gamma, idx)) { // (uniform over the block) nothing to draw: keep its plan entry empty
        if (threadIdx.x == 0 && next.enabled) plan_next_cand(next, j, 0);
        return;
    }
    const float *row = logits + (size_t)j * V;
    float mx;
    int am;
    row_max_argmax(row, V, redv, redi, mx, am);
    if (T == 0.f) {
        if (threadIdx.x == 0) {
            cand[j * gamma + idx] = am;
            if (next.enabled) plan_next_cand(next, j, am);
        }
        return;
    }
    float invT = 1.0f / T;
    float z = row_sumexp(row, V, mx, invT, redv);
    float invZ = 1.0f / z;
    float *qrow = q + ((size_t)j * gamma + idx) * V;
    int nvec = (V + 3) / 4;
    for (int v = threadIdx.x; v < nvec; v += blockDim.x) {
        float4 f = load4_guard(row, v, V, -3.0e38f);
        float4 p;
        p.x = expf((f.x - mx) * invT) * invZ;
        p.y = expf((f.y - mx) * invT) * invZ;
        p.z = expf((f.z - mx) * invT) * invZ;
        p.w = expf((f.w - mx) * invT) * invZ;
        if (4 * v + 3 < V) *(float4 *)(qrow + 4 * v) = p;
        else {
            if (4 * v < V) qrow[4 * v] = p.x;
            if (4 * v + 1 < V) qrow[4 * v + 1] = p.y;
            if (4 * v + 2 < V) qrow[4 * v + 2] = p.z;
        }
    }
    __syncthreads(); // q row of this block is complete and visible to the block
    auto wfun = [&](int v) {
        float4 f = load4_guard(row, v, V, -3.0e38f);
        float4 p;
        p.x = expf((f.x - mx) * invT) * invZ;
        p.y = 4 * v + 1 < V ? expf((f.y - mx) * invT) * invZ : 0.f;
        p.z = 4 * v + 2 < V ? expf((f.z - mx) * invT) * invZ : 0.f;
        p.w = 4 * v + 3 < V ? expf((f.w - mx) * invT) * invZ : 0.f;
        return p;
    };
    int pick = block_pick_cdf(wfun, V, u[j * gamma + idx], &ps, nullptr);
    if (threadIdx.x == 0) {
        cand[j * gamma + idx] = pick;
        if (next.enabled) plan_next_cand(next, j, pick);
    }
}

hipError_t launch_draft_sample(hipStream_t s, const float *logits, int n_seq, int V, float T, const float *u,
                               int gamma, int idx, int32_t *cand, float *q, const NextPlan &next, const float *stats,
                               int stats_nb, int *did_embed)
{
    if (did_embed) *did_embed = 0;
    const int n_slices = (V + DS_SLICE - 1) / DS_SLICE;
    if (stats && stats_nb > 0 && stats_nb * 32 == V && n_slices <= DS_MAX_SLICES && n_seq <= 65535) {
        if (did_embed) *did_embed = next.enabled && next.embed;
        if (T > 0.f)
            hipLaunchKernelGGL(draft_sample_split_kernel, dim3(n_slices, n_seq), dim3(256), 0, s, logits, stats, stats_nb,
                               V, T, u, gamma, idx, cand, q, next);
        else
            hipLaunchKernelGGL(draft_argmax_split_kernel, dim3(n_seq), dim3(256), 0, s, stats, stats_nb, gamma, idx, cand,
                               next);
        return hipGetLastError();
    }
    if (V <= ROW_NSEG * ROW_THREADS * 4)
        hipLaunchKernelGGL(draft_sample_fast_kernel, dim3(n_seq), dim3(ROW_THREADS), 0, s, logits, V, T, u, gamma, idx,
                           cand, q, next);
    else
        hipLaunchKernelGGL(draft_sample_kernel, dim3(n_seq), dim3(1024), 0, s, logits, V, T, u, gamma, idx, cand, q,
                           next);
    return hipGetLastError();
}

// ---------------------------------------------------------------- commit (KV rollback)
__device__ void commit_one(CtxView cv, int b, int gamma, const int32_t *cand_j, int n_acc, int next_tok)
{
    int n = cv.ntok[b];
    int64_t off = cv.off[b];
    int cap = cv.cap[b];
    if (n_acc < 0) n_acc = 0;
    if (n_acc > gamma) n_acc = gamma;
    if (n + n_acc + 1 > cap) {
        atomicOr(cv.status, 1);
        return;
    }
    for (int i = 0; i < n_acc; i++) cv.tokens[off + n + i] = cand_j[i];
    cv.tokens[off + n + n_acc] = next_tok;
    // running estimate of Equation 1's alpha: accepted over examined candidates (a step that rejects at
    // position k has examined k + 1 of them)
    cv.pol[b] += n_acc;
    cv.pol[cv.B + b] += n_acc < gamma ? n_acc + 1 : gamma;
    int nn = n + n_acc + 1;
    cv.ntok[b] = nn;
    for (int sl = 0; sl < cv.n_slots; sl++) {
        int *kv = cv.kvlen + (size_t)sl * cv.B + b;
        if (*kv > nn - 1) *kv = nn - 1;
    }
}

__global__ void commit_kernel(CtxView cv, const int32_t *seq_ids, int n_seq, int gamma, const int32_t *cand,
                              const int32_t *n_acc, const int32_t *next_tok)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_seq) return;
    int b = seq_ids ? seq_ids[j] : j;
    if (b < 0 || b >= cv.B) {
        atomicOr(cv.status, 4);
        return;
    }
    commit_one(cv, b, seq_gamma(cv, b, gamma), cand + (size_t)j * gamma, n_acc[j], next_tok[j]);
}

// Candidate-count policy on the device (Section 1, Equation 1): for each selected sequence, alpha = accepted / examined so
// far (alpha0 before anything was examined) and gamma = the count in [0, gamma_max] that maximises
// (1 - alpha^(gamma+1)) / ((1 - alpha) (gamma c + 1)), the smallest on ties.  Written out operation by operation
// (no fused multiply-add), in the order the host function sd_choose_gamma uses, so both pick the same count.
__global__ void policy_choose_kernel(CtxView cv, const int32_t *seq_ids, int n_seq, double c_ratio, int gamma_max,
                                     double alpha0, int32_t *gamma_all, int32_t *gammas_out)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_seq) return;
    const int b = seq_ids ? seq_ids[j] : j;
    if (b < 0 || b >= cv.B) {
        atomicOr(cv.status, 4);
        if (gammas_out) gammas_out[j] = 0;
        return;
    }
    const int acc = cv.pol[b], exam = cv.pol[cv.B + b];
    const double alpha = exam > 0 ? __ddiv_rn((double)acc, (double)exam) : alpha0;
    int best = 0;
    double best_v = -1.0;
    for (int g = 0; g <= gamma_max; g++) {
        double tokens = 0.0, term = 1.0;
        for (int i = 0; i <= g; i++) {
            tokens = __dadd_rn(tokens, term);
            term = __dmul_rn(term, alpha);
        }
        const double v = __ddiv_rn(tokens, __dadd_rn(__dmul_rn((double)g, c_ratio), 1.0));
        if (v > best_v) best = g, best_v = v;
    }
    gamma_all[b] = best;
    if (gammas_out) gammas_out[j] = best;
}

hipError_t launch_policy_choose(hipStream_t s, CtxView cv, const int32_t *seq_ids, int n_seq, double c_ratio, int gamma_max,
                                double alpha0, int32_t *gamma_all, int32_t *gammas_out)
{
    hipLaunchKernelGGL(policy_choose_kernel, dim3((n_seq + 255) / 256), dim3(256), 0, s, cv, seq_ids, n_seq, c_ratio, gamma_max,
                       alpha0, gamma_all, gammas_out);
    return hipGetLastError();
}

hipError_t launch_commit(hipStream_t s, CtxView cv, const int32_t *seq_ids, int n_seq, int gamma,
                         const int32_t *cand, const int32_t *n_acc, const int32_t *next_tok)
{
    hipLaunchKernelGGL(commit_kernel, dim3((n_seq + 255) / 256), dim3(256), 0, s, cv, seq_ids, n_seq, gamma, cand,
                       n_acc, next_tok);
    return hipGetLastError();
}

// ---------------------------------------------------------------- verify tail
// Fused vocabulary softmax + accept scan + residual + resample, one block per
// sequence.  Row statistics (max, sum of exponentials, argmax) of the gamma+1
// logit rows are block reductions; the accept scan runs on thread 0; only the
// row that decides the next token is traversed again.
__global__ __launch_bounds__(1024) void verify_tail_kernel(const float *logits, int gamma, int V, float T,
                                                           const int32_t *cand, const float *q, const float *u,
                                                           const int32_t *seq_ids, int32_t *n_acc_out,
                                                           int32_t *next_out, int commit, CtxView cv)
{
    __shared__ PickScratch ps;
    __shared__ float redv[32];
    __shared__ int redi[32];
    __shared__ float s_mx[SD_MAX_GAMMA + 1], s_z[SD_MAX_GAMMA + 1];
    __shared__ int s_am[SD_MAX_GAMMA + 1];
    __shared__ int s_nacc;
    __shared__ float s_zr;
    int j = blockIdx.x;
    const float *rows = logits + (size_t)j * (gamma + 1) * V;
    const int32_t *cj = cand + (size_t)j * gamma;
    float invT = T > 0.f ? 1.0f / T : 0.f;
    const int stride_g = gamma; // row slots of the call: strides of cand, q and u
    {   // with per-sequence candidate counts this sequence has gj <= gamma candidates (and gj + 1 live rows)
        const int bb = seq_ids ? seq_ids[j] : j;
        if (cv.gam && bb >= 0 && bb < cv.B) gamma = seq_gamma(cv, bb, gamma);
    }
    for (int i = 0; i <= gamma; i++) {
        float mx;
        int am;
        row_max_argmax(rows + (size_t)i * V, V, redv, redi, mx, am);
        float z = 1.f;
        if (T > 0.f) z = row_sumexp(rows + (size_t)i * V, V, mx, invT, redv);
        if (threadIdx.x == 0) {
            s_mx[i] = mx;
            s_z[i] = z;
            s_am[i] = am;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int n_acc = 0;
        for (int i = 0; i < gamma; i++) {
            int c = cj[i];
            bool ok;
            if (T == 0.f) ok = c == s_am[i];
            else if (c < 0 || c >= V) ok = false;
            else {
                float p = expf((rows[(size_t)i * V + c] - s_mx[i]) * invT) / s_z[i];
                float qc = q[((size_t)j * stride_g + i) * V + c];
                qc = fmaxf(qc, 1.17549435e-38f);
                ok = u[j * (stride_g + 1) + i] < p / qc;
            }
            if (!ok) break;
            n_acc++;
        }
        s_nacc = n_acc;
    }
    __syncthreads();
    int n_acc = s_nacc;
    int next;
    if (T == 0.f) {
        next = s_am[n_acc];
    } else {
        const float *row = rows + (size_t)n_acc * V;
        float mx = s_mx[n_acc], invZ = 1.0f / s_z[n_acc];
        float uu = u[j * (stride_g + 1) + gamma];
        auto pfun = [&](int v) {
            float4 f = load4_guard(row, v, V, -3.0e38f);
            float4 p;
            p.x = expf((f.x - mx) * invT) * invZ;
            p.y = 4 * v + 1 < V ? expf((f.y - mx) * invT) * invZ : 0.f;
            p.z = 4 * v + 2 < V ? expf((f.z - mx) * invT) * invZ : 0.f;
            p.w = 4 * v + 3 < V ? expf((f.w - mx) * invT) * invZ : 0.f;
            return p;
        };
        bool use_p = n_acc >= gamma;
        if (!use_p) {
            const float *qrow = q + ((size_t)j * stride_g + n_acc) * V;
            auto rfun = [&](int v) {
                float4 p = pfun(v);
                float4 qq = load4_guard(qrow, v, V, 0.f);
                return make_float4(fmaxf(p.x - qq.x, 0.f), fmaxf(p.y - qq.y, 0.f), fmaxf(p.z - qq.z, 0.f),
                                   fmaxf(p.w - qq.w, 0.f));
            };
            float zr = 0.f;
            next = block_pick_cdf(rfun, V, uu, &ps, &zr);
            if (threadIdx.x == 0) s_zr = zr;
            __syncthreads();
            if (!(s_zr > 0.f)) use_p = true; // numerically empty residual: draw from p
            __syncthreads();
        }
        if (use_p) next = block_pick_cdf(pfun, V, uu, &ps, nullptr);
    }
    if (threadIdx.x == 0) {
        n_acc_out[j] = n_acc;
        next_out[j] = next;
        if (commit) {
            int b = seq_ids ? seq_ids[j] : j;
            if (b >= 0 && b < cv.B) commit_one(cv, b, gamma, cj, n_acc, next);
            else atomicOr(cv.status, 4);
        }
    }
}

// Same decisions as verify_tail_kernel in two launches.  verify_stats_kernel: one block per logits row
// (n_seq * (gamma + 1) blocks, so the exponentials of the rows run on different compute units), each row
// read once into registers; writes max, z and argmax per row.  verify_decide_kernel: one block per
// sequence; the gamma acceptance tests are evaluated by gamma threads in parallel and scanned by
// thread 0, then the deciding row is read once more for the resample.
__global__ __launch_bounds__(ROW_THREADS) void verify_stats_kernel(const float *logits, int V, float T, float *stats)
{
    __shared__ FastScratch fs;
    RowRegs r;
    row_load(logits + (size_t)blockIdx.x * V, V, -3.0e38f, r);
    float mx, z;
    int am;
    row_stats_regs(r, T > 0.f ? 1.0f / T : 0.f, &fs, mx, am, z);
    if (threadIdx.x == 0) {
        stats[3 * blockIdx.x] = mx;
        stats[3 * blockIdx.x + 1] = z;
        stats[3 * blockIdx.x + 2] = __int_as_float(am);
    }
}

__global__ __launch_bounds__(ROW_THREADS) void verify_decide_kernel(const float *logits, const float *stats, int gamma,
                                                                     int V, float T, const int32_t *cand,
                                                                     const float *q, const float *u,
                                                                     const int32_t *seq_ids, int32_t *n_acc_out,
                                                                     int32_t *next_out, int commit, CtxView cv)
{
    __shared__ FastScratch fs;
    __shared__ int s_ok[SD_MAX_GAMMA];
    __shared__ int s_nacc;
    __shared__ float s_zr;
    const int j = blockIdx.x;
    const float *rows = logits + (size_t)j * (gamma + 1) * V;
    const float *st = stats + (size_t)j * (gamma + 1) * 3;
    const int32_t *cj = cand + (size_t)j * gamma;
    const float invT = T > 0.f ? 1.0f / T : 0.f;
    const int stride_g = gamma; // row slots of the call: strides of cand, q and u
    {   // with per-sequence candidate counts this sequence has gj <= gamma candidates (and gj + 1 live rows)
        const int bb = seq_ids ? seq_ids[j] : j;
        if (cv.gam && bb >= 0 && bb < cv.B) gamma = seq_gamma(cv, bb, gamma);
    }
    if ((int)threadIdx.x < gamma) {
        const int i = threadIdx.x;
        const int c = cj[i];
        bool ok;
        if (T == 0.f) ok = c == __float_as_int(st[3 * i + 2]);
        else if (c < 0 || c >= V) ok = false;
        else {
            const float p = expf((rows[(size_t)i * V + c] - st[3 * i]) * invT) / st[3 * i + 1];
            float qc = q[((size_t)j * stride_g + i) * V + c];
            qc = fmaxf(qc, 1.17549435e-38f);
            ok = u[j * (stride_g + 1) + i] < p / qc;
        }
        s_ok[i] = ok ? 1 : 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int n = 0;
        while (n < gamma && s_ok[n]) n++;
        s_nacc = n;
    }
    __syncthreads();
    const int n_acc = s_nacc;
    int next;
    if (T == 0.f) {
        next = __float_as_int(st[3 * n_acc + 2]);
    } else {
        const float mx = st[3 * n_acc], invZ = 1.0f / st[3 * n_acc + 1];
        const float uu = u[j * (stride_g + 1) + gamma];
        RowRegs r;
        row_load(rows + (size_t)n_acc * V, V, -3.0e38f, r);
#pragma unroll
        for (int it = 0; it < ROW_NSEG; it++) {
            float4 f = r.f[it];
            f.x = expf((f.x - mx) * invT) * invZ;
            f.y = expf((f.y - mx) * invT) * invZ;
            f.z = expf((f.z - mx) * invT) * invZ;
            f.w = expf((f.w - mx) * invT) * invZ;
            r.f[it] = f;
        }
        bool use_p = n_acc >= gamma;
        next = 0;
        if (!use_p) {
            RowRegs w;
            row_load(q + ((size_t)j * stride_g + n_acc) * V, V, 0.f, w);
#pragma unroll
            for (int it = 0; it < ROW_NSEG; it++) {
                w.f[it].x = fmaxf(r.f[it].x - w.f[it].x, 0.f);
                w.f[it].y = fmaxf(r.f[it].y - w.f[it].y, 0.f);
                w.f[it].z = fmaxf(r.f[it].z - w.f[it].z, 0.f);
                w.f[it].w = fmaxf(r.f[it].w - w.f[it].w, 0.f);
            }
            float zr = 0.f;
            next = pick_regs(w, V, uu, &fs, &zr);
            if (threadIdx.x == 0) s_zr = zr;
            __syncthreads();
            if (!(s_zr > 0.f)) use_p = true; // numerically empty residual: draw from p
            __syncthreads();
        }
        if (use_p) next = pick_regs(r, V, uu, &fs, nullptr);
    }
    if (threadIdx.x == 0) {
        n_acc_out[j] = n_acc;
        next_out[j] = next;
        if (commit) {
            const int b = seq_ids ? seq_ids[j] : j;
            if (b >= 0 && b < cv.B) commit_one(cv, b, gamma, cj, n_acc, next);
            else atomicOr(cv.status, 4);
        }
    }
}

hipError_t launch_verify_tail(hipStream_t s, const float *logits, int n_seq, int gamma, int V, float T,
                              const int32_t *cand, const float *q, const float *u, const int32_t *seq_ids,
                              int32_t *n_acc, int32_t *next_tok, int commit, CtxView cv, float *stats)
{
    if (V <= ROW_NSEG * ROW_THREADS * 4 && stats) {
        hipLaunchKernelGGL(verify_stats_kernel, dim3(n_seq * (gamma + 1)), dim3(ROW_THREADS), 0, s, logits, V, T, stats);
        hipLaunchKernelGGL(verify_decide_kernel, dim3(n_seq), dim3(ROW_THREADS), 0, s, logits, stats, gamma, V, T, cand, q,
                           u, seq_ids, n_acc, next_tok, commit, cv);
    } else
        hipLaunchKernelGGL(verify_tail_kernel, dim3(n_seq), dim3(1024), 0, s, logits, gamma, V, T, cand, q, u, seq_ids,
                           n_acc, next_tok, commit, cv);
    return hipGetLastError();
}

// ---------------------------------------------------------------- routing
__global__ void route_kernel(const float *W, const float *b, int n_drafts, int emb, const float *e, int n,
                             int32_t *id)
{
    int i = blockIdx.x;
    int lane = threadIdx.x;
    float best = -3.0e38f;
    int bi = 0;
    for (int k = 0; k < n_drafts; k++) {
        float acc = 0.f;
        for (int t = lane; t < emb; t += WAVE) acc += W[(size_t)k * emb + t] * e[(size_t)i * emb + t];
        acc = wave_sum(acc) + (b ? b[k] : 0.f);
        if (acc > best) {
            best = acc;
            bi = k;
        }
    }
    if (lane == 0) id[i] = bi;
}

hipError_t launch_route(hipStream_t s, const float *W, const float *b, int n_drafts, int emb, const float *e, int n,
                        int32_t *id)
{
    hipLaunchKernelGGL(route_kernel, dim3(n), dim3(WAVE), 0, s, W, b, n_drafts, emb, e, n, id);
    return hipGetLastError();
}

// ---------------------------------------------------------------- synthetic cache load
template <typename T>
__global__ void set_kv_kernel(const T *k_rows, const T *v_rows, int len, int H, int hd, int64_t seq_off,
                              int64_t total_cap, T *Kl, T *Vtl)
{
    size_t n = (size_t)len * H * hd;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        int d = i % hd;
        int h = (i / hd) % H;
        int t = i / ((size_t)hd * H);
        Kl[(size_t)h * total_cap * hd + kt_offset(hd, seq_off + t, d)] = k_rows[i];
        Vtl[(size_t)h * hd * total_cap + vt_offset(hd, seq_off + t, d)] = v_rows[i];
    }
}

hipError_t launch_set_kv(hipStream_t s, int dtype, const void *k_rows, const void *v_rows, int len, int H, int hd,
                         int64_t seq_off, int64_t total_cap, void *Kl, void *Vtl)
{
    size_t n = (size_t)len * H * hd;
    int blocks = (int)((n + 255) / 256);
    if (blocks > 65535) blocks = 65535;
    if (blocks < 1) blocks = 1;
    if (dtype == SD_BF16)
        hipLaunchKernelGGL(set_kv_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t *)k_rows,
                           (const bf16_t *)v_rows, len, H, hd, seq_off, total_cap, (bf16_t *)Kl, (bf16_t *)Vtl);
    else
        hipLaunchKernelGGL(set_kv_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float *)k_rows,
                           (const float *)v_rows, len, H, hd, seq_off, total_cap, (float *)Kl, (float *)Vtl);
    return hipGetLastError();
}

// ---------------------------------------------------------------- measurement helper: a plain streaming read
// Reads `n_vec` 16-byte vectors once and folds them into one word (written only if it hits a magic value, so that
// the loads cannot be dropped): what the memory system gives a kernel that does nothing but read, the practical
// ceiling the weight-streaming GEMMs are held against.  NT = false: grid-strided, ordinary loads; NT = true: every
// block reads one contiguous range with the nontemporal hint, eight loads in flight per thread - the fastest
// pattern found on this part (1 GiB: 7.0 against 5.4-6.3 TB/s).
typedef __attribute__((ext_vector_type(4))) unsigned int sr_u32x4;
template <bool NT, bool FOLD>
__global__ __launch_bounds__(256) void stream_read_kernel(const sr_u32x4 *__restrict__ p, size_t n_vec, uint32_t *out)
{
    constexpr int U = NT ? 8 : 4;
    size_t i, stride, end;
    if (NT) {
        const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
        i = (size_t)blockIdx.x * per + threadIdx.x;
        stride = 256;
        end = min(n_vec, (size_t)(blockIdx.x + 1) * per);
    } else {
        i = (size_t)blockIdx.x * 256 + threadIdx.x;
        stride = (size_t)gridDim.x * 256;
        end = n_vec;
    }
    uint32_t acc = 0;
    for (; i + (U - 1) * stride < end; i += U * stride) {
        sr_u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; u++) v[u] = ld_stream<NT>(p + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; u++) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < end; i += stride) {
        const sr_u32x4 a = ld_stream<NT>(p + i);
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (FOLD) { // checking mode: XOR of every word read, accumulated into out[0] (one atomic per wave)
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o, 64);
        if ((threadIdx.x & 63) == 0) atomicXor(out, acc);
    } else if (acc == 0x9e3779b9u) {
        out[0] = acc;
    }
}

int g_stream_read_nt = 1; // option "stream_read_nt"
hipError_t launch_stream_read(hipStream_t s, const void *buf, size_t bytes, uint32_t *out)
{
    const sr_u32x4 *p = (const sr_u32x4 *)buf;
    const size_t n_vec = bytes / 16;
    switch ((g_stream_read_nt & 1) | (g_stream_read_nt & 2)) { // bit 1: checking mode (XOR of all words into *out)
    case 0: hipLaunchKernelGGL((stream_read_kernel<false, false>), dim3(2048), dim3(256), 0, s, p, n_vec, out); break;
    case 1: hipLaunchKernelGGL((stream_read_kernel<true, false>), dim3(2048), dim3(256), 0, s, p, n_vec, out); break;
    case 2: hipLaunchKernelGGL((stream_read_kernel<false, true>), dim3(2048), dim3(256), 0, s, p, n_vec, out); break;
    default: hipLaunchKernelGGL((stream_read_kernel<true, true>), dim3(2048), dim3(256), 0, s, p, n_vec, out); break;
    }
    return hipGetLastError();
}
