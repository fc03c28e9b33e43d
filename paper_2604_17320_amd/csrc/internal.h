// Host-side launchers shared between translation units of libquota (not part
// of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include "../../include/quota.h"

// score kernel with a separate sequence stride for the sumsq/ressq arrays, so
// the layer can pass the per-row side outputs of the quantizer directly
int quota_internal_score(const float *sumsq, const float *ressq, long stride_sq,
                         const float *cm_inter, const float *cm_intra, int B, int Nv,
                         const quota_score_params *p, float *score, float *normed, hipStream_t st);

struct quota_compact_args {
    int B, N, vis_begin, Nv, k_keep, n_keep, d;
    const int32_t *keep_idx;
    const void *x, *o;
    const int32_t *pos;
    const void *skc, *sks, *svc, *svs;     // staged 4-bit K/V of all N rows
    void *x_out, *o_out;
    int32_t *pos_out, *rows_out;
    quota_kv_cache *cache;
};
int quota_internal_compact(const quota_compact_args *a, hipStream_t st);

int quota_internal_vector_metrics(const void *v_f16, int B, int Nv, int d, int ldv, long stride_b,
                                  float *sumsq, float *ressq, hipStream_t st);
