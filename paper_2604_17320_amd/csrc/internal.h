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

// score + top-k of the min(K, Nv) best tokens in one launch; cues either head-averaged
// (cm_inter / cm_intra) or per head (partial [B][H][Nv][2], head mean taken in the kernel)
int quota_internal_score_topk(const float *sumsq, const float *ressq, long stride_sq,
                              const float *cm_inter, const float *cm_intra, const float *partial,
                              int H, float *cm_out_inter, float *cm_out_intra, int B, int Nv,
                              const quota_score_params *p, float *score, int K, int32_t *keep_idx,
                              hipStream_t st);

// attention + per-head column masses; partial_out (optional) [B][H][Nv][2] in the workspace
int quota_internal_attention(const void *q_f16, const void *khat_f16, const void *vhat_f16, int B,
                             int N, int H, int Hkv, int dh, int vis_begin, int Nv, void *o_f16,
                             bool want_cues, void *ws, const float **partial_out, hipStream_t st);

struct quota_compact_args {
    int B, N, vis_begin, Nv, k_keep, n_keep, d, dkv;      // dkv: width of a K or V row (Hkv * dh)
    const int32_t *keep_idx;              // null: the first k_keep visual tokens (k_keep = Nv: all of them)
    const void *x, *o;
    const int32_t *pos;
    const void *skc, *sks, *svc, *svs;     // staged 4-bit K/V of all N rows
    void *x_out, *o_out;                   // o_out optional (fp16 copy of the kept attention rows)
    uint8_t *oq_out;                       // optional: packed int4 codes of the kept attention rows ...
    float *os_out;                         // ... and their per-token scales (the quantizer Q)
    int32_t *pos_out, *rows_out;
    quota_kv_cache *cache;
};
// Appends at row cache->len but does not advance it.
int quota_internal_compact(const quota_compact_args *a, hipStream_t st);

int quota_internal_vector_metrics(const void *v_f16, int B, int Nv, int d, int ldv, long stride_b,
                                  float *sumsq, float *ressq, hipStream_t st);

// Moves the B staged (dense) 4-bit K/V rows of a decode step to row cache->len of each
// sequence (the caller advances cache->len).  QUOTA_ERR_CAPACITY if the cache is full.
int quota_internal_kv_append_rows(int d, const uint8_t *skc, const void *sks, const uint8_t *svc,
                                  const void *svs, quota_kv_cache *cache, hipStream_t st);

// Arguments of the fused QKV epilogue: what quota_rope_kv_quant takes, minus the qkv input.
struct quota_qkv_epilogue {
    const int32_t *pos;
    const float *cosT, *sinT;
    int n_pos, d, dkv, dh;                  // q width H*dh, K/V width Hkv*dh
    f16 *q_rot, *khat, *vhat;
    uint32_t *k_codes, *v_codes;
    f16 *k_scales, *v_scales;
    long code_row_stride, code_row_offset;   // codes / scales of token row m go to row m * stride + offset
    const int32_t *row_step;                 // optional (device): ... + clamp(*row_step, 0, max_steps - 1)
    int max_steps;
};
int quota_internal_w4a4_gemm_qkv(const uint8_t *qa, const float *sa, int M, const quota_weights *W,
                                 void *y_opt, const quota_qkv_epilogue *qe, hipStream_t st);

// quota_rope_kv_quant with Hkv K/V heads: qkv rows are q (H*dh) | k (Hkv*dh) | v (Hkv*dh).
int quota_internal_rope_kv_quant(const void *qkv_f16, int M, int H, int Hkv, int dh, const int32_t *pos,
                                 const float *cosT, const float *sinT, int n_pos, void *q_rot_f16,
                                 void *khat_f16, void *vhat_f16, uint8_t *k_codes, void *k_scales,
                                 uint8_t *v_codes, void *v_scales, hipStream_t st);

// *step_dev += 1 (one thread; capturable)
int quota_internal_advance_step(int32_t *step_dev, hipStream_t st);


// Limits that the kernels behind the layer calls enforce, for the up-front checks of the layer
// calls (a call that returns an error must not have enqueued anything).
#define QUOTA_MAX_SCORED_TOKENS 8192      // visual tokens per sequence the score / top-k kernel holds in LDS
#define QUOTA_MAX_DECODE_ROWS 8192        // cached rows per sequence the decode attention softmaxes over
#define QUOTA_MAX_MODEL_WIDTH 16384       // d: the compaction gather keeps a row in registers
#define QUOTA_MAX_ROW_COLS 32768          // widest row of the row quantizers (the FFN width F)
