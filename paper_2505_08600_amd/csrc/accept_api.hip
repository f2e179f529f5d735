// The acceptance rule as a call of its own (Section 3.1: speculative-sampling verification; greedy as its
// argmax limit): vocabulary softmax + accept scan + residual + resample on logits the caller already has.
// sd_verify runs the same kernels behind the target's forward; here they are reachable without a model or a
// context, which is also how the stage is measured alone.
#include <string.h>

#include <mutex>

#include "sd_internal.h"

static int check_accept(const char *who, const float *logits, int n_seq, int gamma, int vocab, float T,
                        const int32_t *cand, const float *q, const float *u, const int32_t *n_acc, const int32_t *next)
{
    if (!logits || !n_acc || !next) return sd_fail(SD_EINVAL, std::string(who) + ": null logits or output");
    if (n_seq < 1) return sd_fail(SD_EINVAL, std::string(who) + ": n_seq < 1");
    if (gamma < 0 || gamma > SD_MAX_GAMMA) return sd_fail(SD_ECAP, std::string(who) + ": gamma must be in [0, 15]");
    if (vocab < 4 || vocab % 4 != 0 || vocab > 262144)
        return sd_fail(SD_EINVAL, std::string(who) + ": vocab must be a multiple of 4 in [4, 262144]");
    if (!(T >= 0.f)) return sd_fail(SD_EINVAL, std::string(who) + ": negative temperature");
    if (gamma > 0 && !cand) return sd_fail(SD_EINVAL, std::string(who) + ": null cand");
    if (T > 0.f && (!u || (gamma > 0 && !q))) return sd_fail(SD_EINVAL, std::string(who) + ": sampling needs uniforms and q");
    if (((uintptr_t)logits & 15) || ((uintptr_t)q & 15)) return sd_fail(SD_EINVAL, std::string(who) + ": logits and q must be 16-byte aligned");
    return SD_OK;
}

static int run_accept(const char *who, const float *logits, int n_seq, int gamma, int vocab, float T, const int32_t *cand,
                      const float *q, const float *u, int32_t *n_acc, int32_t *next, float *stats, hipStream_t s)
{
    CtxView none;
    memset(&none, 0, sizeof(none));
    hipError_t e = launch_verify_tail(s, logits, n_seq, gamma, vocab, T, cand, q, u, nullptr, n_acc, next, 0, none, stats);
    if (e != hipSuccess) return sd_fail(SD_EHIP, std::string(who) + ": " + hipGetErrorString(e));
    return SD_OK;
}

extern "C" int sd_accept(const float *logits, int32_t n_seq, int32_t gamma, int32_t vocab, float temperature,
                         const int32_t *cand, const float *q, const float *uniforms, int32_t *n_accepted,
                         int32_t *next_token, float *workspace, void *stream)
{
    int rc = check_accept("sd_accept", logits, n_seq, gamma, vocab, temperature, cand, q, uniforms, n_accepted, next_token);
    if (rc) return rc;
    if (!workspace) return sd_fail(SD_EINVAL, "sd_accept: null workspace");
    return run_accept("sd_accept", logits, n_seq, gamma, vocab, temperature, cand, q, uniforms, n_accepted, next_token,
                      workspace, (hipStream_t)stream);
}

// ---------------------------------------------------------------- the same call without any allocation
// For callers that cannot allocate or carry a workspace (code under graph capture, tight serving loops):
// the per-row statistics that sd_accept passes between its two kernels through `workspace` live in a
// file-scope device array instead.  Every device the library runs on holds its own copy of the array at
// its own address for the life of the process; the address is looked up once per device and kept.
#define SD_ACCEPT_STATIC_MAX_ROWS 4096 // n_seq * (gamma + 1); 48 KiB of device memory per GPU
#define SD_MAX_DEVICES 64
static __device__ __align__(256) float scratch[3 * SD_ACCEPT_STATIC_MAX_ROWS];

static std::mutex g_scratch_mutex;
static float *g_scratch_ptr[SD_MAX_DEVICES]; // device address of `scratch` per device, nullptr until first use

// Device address of this device's copy of `scratch` (the array's name is only a host-side handle).
static int scratch_on_current_device(float **out)
{
    int dev = -1;
    SD_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= SD_MAX_DEVICES) return sd_fail(SD_EINVAL, "sd_accept_static: device ordinal above 63");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        SD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return sd_fail(SD_EHIP, "sd_accept_static: hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = (float *)p;
    }
    *out = g_scratch_ptr[dev];
    return SD_OK;
}

extern "C" int sd_accept_static(const float *logits, int32_t n_seq, int32_t gamma, int32_t vocab, float temperature,
                                const int32_t *cand, const float *q, const float *uniforms, int32_t *n_accepted,
                                int32_t *next_token, void *stream)
{
    int rc = check_accept("sd_accept_static", logits, n_seq, gamma, vocab, temperature, cand, q, uniforms, n_accepted,
                          next_token);
    if (rc) return rc;
    if ((int64_t)n_seq * (gamma + 1) > SD_ACCEPT_STATIC_MAX_ROWS)
        return sd_fail(SD_ECAP, "sd_accept_static: n_seq * (gamma + 1) exceeds 4096 rows (use sd_accept with a workspace)");
    float *stats = nullptr;
    rc = scratch_on_current_device(&stats);
    if (rc) return rc;
    // (nothing to clear: the first kernel writes all 3 * n_seq * (gamma + 1) entries the second one reads)
    return run_accept("sd_accept_static", logits, n_seq, gamma, vocab, temperature, cand, q, uniforms, n_accepted,
                      next_token, stats, (hipStream_t)stream);
}
