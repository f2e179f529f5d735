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
