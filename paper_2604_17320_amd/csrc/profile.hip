// Per-kernel event timing for the benchmark (see profile.h).
#include "profile.h"
#include <stdlib.h>

QuotaProfiler g_quota_prof;

static const char *const kKernelNames[QUOTA_KERNEL_COUNT] = {
    "quantize_act", "rmsnorm_quantize_act", "silu_mul_quantize_act", "w4a4_gemm_64x256",
    "w4a4_gemm_64x128", "w4a4_gemm_32x128", "w4a4_gemm_32x128_deep", "w4a4_gemm_64x128_lean", "w4a4_gemm_other", "rope_kv_quant", "kv_quant_append", "attention_fwd",
    "attention_colmass", "score_tokens", "topk_prune", "compact_rows", "quantize_weights",
    "pack_weights", "attention_decode", "kv_append_rows", "w4a4_gemm_rows16"};

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
    if (!p.ev || !p.kid || !p.ops || !p.bytes) {
        free(p.ev); free(p.kid); free(p.ops); free(p.bytes);
        p = QuotaProfiler();
        return QUOTA_ERR_INVALID_ARG;
    }
    for (int i = 0; i < 2 * max_launches; ++i)
        if (hipEventCreate(&p.ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(p.ev[j]);      // exactly the events created
            free(p.ev); free(p.kid); free(p.ops); free(p.bytes);
            p = QuotaProfiler();
            return QUOTA_ERR_HIP;
        }
    p.cap = max_launches;
    p.used = 0;
    p.on = true;
    return QUOTA_OK;
}

namespace {
__global__ void empty_kernel() {}
}

static int bracket_median(int reps, int kernels, hipStream_t st, hipEvent_t *ev, float *ms, float *out)
{
    for (int i = 0; i < reps; ++i) {
        (void)hipEventRecord(ev[2 * i], st);
        for (int k = 0; k < kernels; ++k) empty_kernel<<<1, 64, 0, st>>>();
        (void)hipEventRecord(ev[2 * i + 1], st);
    }
    for (int i = 0; i < reps; ++i)
        if (hipEventSynchronize(ev[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms[i], ev[2 * i], ev[2 * i + 1]) != hipSuccess)
            return QUOTA_ERR_HIP;
    for (int i = 1; i < reps; ++i)           // insertion sort: reps is small
        for (int j = i; j > 0 && ms[j] < ms[j - 1]; --j) { float t = ms[j]; ms[j] = ms[j - 1]; ms[j - 1] = t; }
    *out = ms[reps / 2];
    return QUOTA_OK;
}

extern "C" int quota_profile_bracket_ms(int reps, void *stream, float *bracket_ms, float *empty_kernel_ms)
{
    if (!bracket_ms) return QUOTA_ERR_NULL;
    if (reps <= 0 || reps > 1024) return QUOTA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t *ev = (hipEvent_t *)calloc(2 * (size_t)reps, sizeof(hipEvent_t));
    float *ms = (float *)calloc(reps, sizeof(float));
    if (!ev || !ms) { free(ev); free(ms); return QUOTA_ERR_INVALID_ARG; }
    int rc = QUOTA_OK, made = 0;
    for (; made < 2 * reps; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) { rc = QUOTA_ERR_HIP; break; }
    float t1 = 0.0f, t2 = 0.0f;
    if (rc == QUOTA_OK) rc = bracket_median(reps, 1, st, ev, ms, &t1);
    if (rc == QUOTA_OK) rc = bracket_median(reps, 2, st, ev, ms, &t2);
    if (rc == QUOTA_OK) {
        float one = t2 - t1;                     // what one more empty kernel adds
        *bracket_ms = t1 - one > 0.0f ? t1 - one : 0.0f;
        if (empty_kernel_ms) *empty_kernel_ms = one;
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    free(ev); free(ms);
    return rc;
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
