// Per-kernel event timing for the benchmark (see profile.h).
#include "profile.h"
#include <stdlib.h>

QuotaProfiler g_quota_prof;

static const char *const kKernelNames[QUOTA_KERNEL_COUNT] = {
    "quantize_act", "rmsnorm_quantize_act", "silu_mul_quantize_act", "w4a4_gemm_64x256",
    "w4a4_gemm_64x128", "w4a4_gemm_32x128", "w4a4_gemm_other", "rope_kv_quant", "kv_quant_append", "attention_fwd",
    "attention_colmass", "score_tokens", "topk_prune", "compact_rows", "quantize_weights",
    "pack_weights"};

extern "C" const char *quota_kernel_name(int kernel_id)
{
    return kernel_id >= 0 && kernel_id < QUOTA_KERNEL_COUNT ? kKernelNames[kernel_id] : "?";
}

static void prof_free()
{
    QuotaProfiler &p = g_quota_prof;
    for (int i = 0; i < 2 * p.cap; ++i) (void)hipEventDestroy(p.ev[i]);
    free(p.ev); free(p.kid); free(p.ops); free(p.bytes);
    p = QuotaProfiler();
}

extern "C" int quota_profile_begin(int max_launches)
{
    if (max_launches <= 0 || max_launches > (1 << 20)) return QUOTA_ERR_INVALID_ARG;
    if (g_quota_prof.cap) prof_free();
    QuotaProfiler &p = g_quota_prof;
    p.ev = (hipEvent_t *)calloc(2 * (size_t)max_launches, sizeof(hipEvent_t));
    p.kid = (int *)calloc(max_launches, sizeof(int));
    p.ops = (double *)calloc(max_launches, sizeof(double));
    p.bytes = (double *)calloc(max_launches, sizeof(double));
    if (!p.ev || !p.kid || !p.ops || !p.bytes) return QUOTA_ERR_INVALID_ARG;
    p.cap = max_launches;
    for (int i = 0; i < 2 * max_launches; ++i)
        if (hipEventCreate(&p.ev[i]) != hipSuccess) { p.cap = i / 2; prof_free(); return QUOTA_ERR_HIP; }
    p.used = 0;
    p.on = true;
    return QUOTA_OK;
}

extern "C" int quota_profile_collect(quota_kernel_stat *stats)
{
    QuotaProfiler &p = g_quota_prof;
    if (!stats) return QUOTA_ERR_NULL;
    if (!p.cap) return QUOTA_ERR_INVALID_ARG;
    p.on = false;
    for (int k = 0; k < QUOTA_KERNEL_COUNT; ++k) {
        stats[k].launches = 0; stats[k].total_ms = 0; stats[k].ops = 0; stats[k].bytes = 0;
    }
    int rc = QUOTA_OK;
    for (int i = 0; i < p.used; ++i) {
        float ms = 0.0f;
        if (hipEventSynchronize(p.ev[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, p.ev[2 * i], p.ev[2 * i + 1]) != hipSuccess) { rc = QUOTA_ERR_HIP; break; }
        quota_kernel_stat &s = stats[p.kid[i]];
        s.launches += 1; s.total_ms += ms; s.ops += p.ops[i]; s.bytes += p.bytes[i];
    }
    prof_free();
    return rc;
}
