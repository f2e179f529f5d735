#include "sd_internal.h"
hipError_t launch_gemm_skinny_bf16(hipStream_t, int, const void *, WeightSeg, int, int, int, float *, void *) { return hipErrorNotSupported; }
hipError_t launch_attn_mfma_bf16(hipStream_t, const void *, const void *, const void *, PlanView, CtxView, int, int, int, int, int64_t, int, float *, size_t, void *) { return hipErrorNotSupported; }
