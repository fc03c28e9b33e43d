/*
 * libquota -- C ABI of the MI355X (gfx950) implementation of the QUOTA hot
 * path: a W4A4 language-model prefill layer that scores, top-k prunes and
 * compacts visual tokens inside the layer and writes a 4-bit KV cache.
 *
 * General rules
 *   - Every pointer named in a signature is a DEVICE pointer owned by the
 *     caller unless it is marked "host".  The library allocates no device
 *     memory; scratch comes from a caller workspace whose size the
 *     *_workspace_bytes call reports.
 *   - Descriptor structs (quota_weights, quota_kv_cache, quota_layer,
 *     quota_state, quota_score_params, quota_taps) live in HOST memory.
 *   - `stream` is a hipStream_t passed as void*.  Calls only enqueue work on
 *     that stream; none synchronises.  Calls on one stream are ordered.
 *   - Every call returns QUOTA_OK or a negative error code and enqueues
 *     nothing when it returns an error.  No exceptions cross the boundary.
 *   - fp16 = IEEE binary16.  int4 data is two's complement, two codes per
 *     byte, element 2j in bits 0-3 and element 2j+1 in bits 4-7.
 *   - Weight groups are 128 input channels (QUOTA_GROUP_W), KV groups are 64
 *     channels of one head (QUOTA_GROUP_KV).
 */
#ifndef QUOTA_H
#define QUOTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QUOTA_GROUP_W 128
#define QUOTA_GROUP_KV 64

enum {
    QUOTA_OK = 0,
    QUOTA_ERR_NULL = -1,        /* a required pointer is null                      */
    QUOTA_ERR_INVALID_ARG = -2, /* negative size, bad flag, bad percentile ...     */
    QUOTA_ERR_SHAPE = -3,       /* shape the kernels do not support (see each call) */
    QUOTA_ERR_CAPACITY = -4,    /* KV cache or workspace too small                 */
    QUOTA_ERR_HIP = -5          /* the HIP runtime reported a launch error         */
};

const char *quota_strerror(int code);
int quota_version(void);

/* ---- W4 weights (unified low-bit execution form, Method overview) ------- */

/* One packed W4 matrix y = x W^T, W logically [N][K].  `packed` holds the
 * int4 codes in the library's GEMM layout ([K/128 groups][N rows][64 bytes],
 * K zero-padded to a multiple of 128), `scales` the fp16 group scales in
 * [group][N] order.  Both buffers are caller-allocated device memory of
 * quota_weights_packed_bytes / quota_weights_scale_bytes bytes. */
typedef struct quota_weights {
    int N;
    int K;
    void *packed;
    void *scales;
} quota_weights;

size_t quota_weights_packed_bytes(int N, int K);
size_t quota_weights_scale_bytes(int N, int K);

/* Symmetric int4 group quantization of an fp32 matrix w [N][K] (row-major,
 * device): per (row, 128-channel group) a = max|w|, scale = fp16(a/7) (1 when
 * that is zero), code = clamp(rne(w / scale), -8, 7).  Writes plain row-major
 * outputs: codes int8 [N][K] (one code per byte) and scales fp16
 * [N][ceil(K/128)].  Requires N, K > 0. */
int quota_quantize_weights(const float *w, int N, int K, int8_t *codes,
                           void *scales_f16, void *stream);

/* Repack plain row-major codes (int8, one per byte, values in [-8,7]) and
 * scales (fp16 [N][ceil(K/128)]) into W->packed / W->scales.  Requires
 * N % 64 == 0 and K % 32 == 0 (QUOTA_ERR_SHAPE otherwise). */
int quota_pack_weights(const int8_t *codes, const void *scales_f16,
                       const quota_weights *W, void *stream);

/* ---- per-token int4 activation quantizer (the quantizer Q of Eq. 6) ----- */

/* x fp16 [M][d] with row stride ldx (elements).  Per row: a = max|x|,
 * scale = a/7 (fp32; 1 if a == 0), code = clamp(rne(x * (7/a)), -8, 7).
 * q_packed uint8 [M][d/2]; scale fp32 [M].  Optional side outputs per row:
 * sumsq_opt = sum x^2 (m_mag^2) and ressq_opt = sum (code*scale - x)^2
 * (m_res^2), both accumulated in fp64 and rounded to fp32.
 * Requires d % 8 == 0, d <= 32768, ldx >= d and ldx % 8 == 0. */
int quota_quantize_act(const void *x_f16, int M, int d, int ldx,
                       uint8_t *q_packed, float *scale, float *sumsq_opt,
                       float *ressq_opt, void *stream);

/* Fused RMSNorm + quantizer used in front of the QKV and gate/up GEMMs:
 * h = fp16((x * rsqrt(mean(x^2) + eps)) * gamma), then the quantizer above
 * applied to h.  The side outputs refer to the RAW row x (the hidden state
 * entering the layer, which is the v_i of Eq. 6): sumsq_opt = sum x^2,
 * ressq_opt = residual of quantizing x itself.  h_opt (fp16 [M][d]) receives
 * the normalised row when not null.  gamma is fp32 [d]. */
int quota_rmsnorm_quantize_act(const void *x_f16, int M, int d, int ldx,
                               const float *gamma, float eps,
                               uint8_t *q_packed, float *scale,
                               float *sumsq_opt, float *ressq_opt,
                               void *h_opt, void *stream);

/* Fused SwiGLU product + quantizer in front of the down projection:
 * z = fp16(silu(gate) * up) with gate = gu[:, 0:F], up = gu[:, F:2F]
 * (gu fp16 [M][2F] dense), then the quantizer applied to z.  z_opt receives
 * z; z_inject_opt, when not null, replaces the computed z (parity harness).
 * Requires F % 8 == 0 and F <= 32768. */
int quota_silu_mul_quantize_act(const void *gu_f16, int M, int F,
                                uint8_t *q_packed, float *scale, void *z_opt,
                                const void *z_inject_opt, void *stream);

/* ---- W4A4 GEMM (W4A4 linear operators of the language model) ------------ */

/* y[m][n] = fp16( sa[m] * sum_g sw[n][g] * acc_g[m][n]  (+ residual[m][n]) ),
 * acc_g the exact int32 dot product of the int4 codes over group g; groups
 * are combined in fp32 with one fused multiply-add each, in ascending order.
 * qa uint8 [M][K/2] packed (row stride K/2), sa fp32 [M], y fp16 [M][ldy],
 * residual_opt fp16 [M][ldr].  acc_i32_opt int32 [M][N] (dense) receives the
 * exact full-K integer dot product (parity harness; slower kernel).
 * Requires M >= 0, ldy >= N; W as accepted by quota_pack_weights. */
int quota_w4a4_gemm(const uint8_t *qa, const float *sa, int M,
                    const quota_weights *W, void *y_f16, int ldy,
                    const void *residual_opt, int ldr, int32_t *acc_i32_opt,
                    void *stream);

/* Pins the GEMM kernel variant that quota_w4a4_gemm and the layer calls use
 * from now on (process-wide; for tests and tuning): -1 = chosen per launch
 * (default); 0..4 = the workgroup-tiled kernels 64x256, 64x128, 32x128,
 * 32x128 deep prefetch, 64x128 lean.  Launches a variant cannot take (at
 * most 16 rows, the int32 output, the 256-column tile with the fused QKV
 * epilogue) ignore the pin.  QUOTA_ERR_INVALID_ARG for other values. */
int quota_set_gemm_variant(int variant);

/* ---- RoPE + 4-bit KV quantization (quantized KV cache) ------------------ */

/* 4-bit KV cache of ONE layer.  Row r of sequence b lives at index
 * b*capacity + r.  k_codes/v_codes uint8 [B][capacity][H*dh/2];
 * k_scales/v_scales fp16 [B][capacity][H*dh/64].  `len` (host field, same
 * for every sequence) is advanced by the append calls. */
typedef struct quota_kv_cache {
    int B, capacity, H, dh;
    int len;
    uint8_t *k_codes;
    void *k_scales;
    uint8_t *v_codes;
    void *v_scales;
    /* Decode loops captured in a HIP graph cannot read a host field that
     * changes from step to step.  When step_dev (device int32, one value) is
     * not null, the decode calls take the cache length as len + *step_dev,
     * read by the kernels: quota_decode_layer appends at that row and does NOT
     * advance len, quota_attention_decode(_gqa) attends over len + *step_dev
     * + 1 rows.  The host checks len + max_steps <= capacity when the call is
     * made and the kernels clamp *step_dev to [0, max_steps - 1].  The caller
     * advances *step_dev between steps (quota_advance_step, capturable) and
     * folds the steps into len when the loop ends.  Null: len alone counts. */
    const int32_t *step_dev;
    int max_steps;
} quota_kv_cache;

/* Rotates q and k (rotate-half pairing (i, i+dh/2)) by the angle tables
 * cosT/sinT (fp32 [n_pos][dh/2]) at each token's ORIGINAL position id
 * pos[row] -- positions stay aligned with tokens after pruning (compaction
 * paragraph after Eq. 9) -- then quantizes k (post-RoPE, rounded to fp16) and
 * v per (token, head, 64-channel group): a = max|x|, s = fp16(a/7) (1 if
 * zero), code = clamp(rne(x * (1/s)), -8, 7).
 * qkv fp16 [M][3*H*dh] (q | k | v), pos int32 [M] with 0 <= pos < n_pos.
 * Outputs for all M rows: q_rot fp16 [M][H*dh]; khat / vhat fp16 [M][H*dh] =
 * fp16(code * s), the values attention sees; staged codes uint8 [M][H*dh/2]
 * and scales fp16 [M][H*dh/64] for k and v.  Requires dh == 64 or 128. */
int quota_rope_kv_quant(const void *qkv_f16, int M, int H, int dh,
                        const int32_t *pos, const float *cosT,
                        const float *sinT, int n_pos, void *q_rot_f16,
                        void *khat_f16, void *vhat_f16, uint8_t *k_codes,
                        void *k_scales, uint8_t *v_codes, void *v_scales,
                        void *stream);

/* Quantizes the rows keep_rows[b][0..n_keep) of k and v (fp16 [B][N][H*dh],
 * k already rotated) exactly as above and appends them to `cache` at row
 * cache->len, then advances cache->len by n_keep.  keep_rows int32
 * [B][n_keep] (device) are row indices inside each sequence; null means rows
 * 0..n_keep-1.  K/V are stored for retained tokens only.
 * QUOTA_ERR_CAPACITY if len + n_keep > capacity (nothing is written). */
int quota_kv_quant_append(const void *k_f16, const void *v_f16, int B, int N,
                          int H, int dh, const int32_t *keep_rows, int n_keep,
                          quota_kv_cache *cache, void *stream);

/* ---- attention over the 4-bit K/V + column masses (Eq. 6 cues) ---------- */

size_t quota_attention_workspace_bytes(int B, int N, int H, int dh);

/* Causal softmax attention of q (fp16 [B][N][H*dh], rotated) over khat / vhat
 * (fp16 [B][N][H*dh], the dequantized 4-bit K/V of the same rows), scores
 * scaled by 1/sqrt(dh), fp16 MFMA with fp32 softmax.  o fp16 [B][N][H*dh].
 * Also the two attention cues of Eq. 6 for each visual key i in
 * [vis_begin, vis_begin+Nv): cm_inter[b][i] = mean over heads of the total
 * probability that text queries put on key i, cm_intra the same for visual
 * queries (fp32 [B][Nv]); pass both null to skip the cue pass.
 * ws: quota_attention_workspace_bytes bytes.  Requires dh == 64 or 128. */
int quota_attention_prefill(const void *q_f16, const void *khat_f16,
                            const void *vhat_f16, int B, int N, int H, int dh,
                            int vis_begin, int Nv, void *o_f16,
                            float *cm_inter, float *cm_intra, void *ws,
                            void *stream);

/* The same with grouped-query attention (the paper's second model family):
 * q and o have H heads per row, khat / vhat have Hkv (rows of Hkv*dh), query
 * head h reads K/V head h / (H/Hkv); the cues average over the H query heads.
 * Requires H % Hkv == 0. */
int quota_attention_prefill_gqa(const void *q_f16, const void *khat_f16,
                                const void *vhat_f16, int B, int N, int H, int Hkv,
                                int dh, int vis_begin, int Nv, void *o_f16,
                                float *cm_inter, float *cm_intra, void *ws,
                                void *stream);

/* For callers that cannot allocate device memory or carry a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): quota_attention_prefill_gqa with its two intermediates (row
 * log-sum-exp, per-head column masses) in a device array that is part of the
 * library image instead of `ws`.  Calls no allocating routine.  Same
 * arguments, results and errors otherwise; additionally QUOTA_ERR_CAPACITY
 * when B*H*N > QUOTA_ATTENTION_STATIC_MAX_ROWS (the array is 12 bytes per
 * (sequence, head, token): 3 MiB, held by every GPU the library runs on until
 * the process ends).  The first call on a device looks the array's address up
 * (once per device; make that call outside graph capture).  All calls on one
 * GPU share the array: calls that overlap on one GPU (different streams or
 * threads) race; calls ordered on one stream do not. */
#define QUOTA_ATTENTION_STATIC_MAX_ROWS 262144
int quota_attention_prefill_static(const void *q_f16, const void *khat_f16,
                                   const void *vhat_f16, int B, int N, int H,
                                   int Hkv, int dh, int vis_begin, int Nv,
                                   void *o_f16, float *cm_inter, float *cm_intra,
                                   void *stream);

/* ---- scoring (Eq. 6-8) and budgeted top-k (Eq. 5, Eq. 9) ---------------- */

typedef struct quota_score_params {
    float w_m, w_c, w_s, w_r; /* weights of mag, inter, intra, res (Eq. 8)   */
    int pct_lo, pct_hi;       /* percentiles of the robust normalisation G   */
} quota_score_params;

/* Table 5 default row: inter 45 %, mag 25 %, intra 10 %, quant 20 %;
 * percentiles 10 / 90. */
void quota_score_params_default(quota_score_params *p);

/* Composite score of every visual token from the four Eq. 6 metrics given as
 * arrays [B][Nv] fp32: sumsq (= m_mag^2) and ressq (= m_res^2) as produced by
 * the quantizer's side outputs, cm_inter and cm_intra as produced by the
 * attention call.  Per sequence and metric, G (Eq. 7) clips to the
 * nearest-rank percentiles (rank = (p*(Nv-1)+50)/100 on the ascending order)
 * and rescales to [0,1] (0.5 for a flat metric); then
 * score = ((w_m*g_mag + w_c*g_inter) + w_s*g_intra) + w_r*g_res in fp32.
 * normed_opt receives the normalised metrics [4][B][Nv] (mag, inter, intra,
 * res).  Requires 0 <= pct_lo <= pct_hi <= 100, Nv <= 8192. */
int quota_score_tokens(const float *sumsq, const float *ressq,
                       const float *cm_inter, const float *cm_intra, int B,
                       int Nv, const quota_score_params *p, float *score,
                       float *normed_opt, void *stream);

/* Same score, with the two vector metrics computed here from the visual
 * token representations v fp16 [B][Nv][d] (row stride ldv, sequence stride
 * stride_b, both in elements).  ws: 2*B*Nv floats. */
int quota_score_tokens_from_hidden(const void *v_f16, int B, int Nv, int d,
                                   int ldv, long stride_b,
                                   const float *cm_inter,
                                   const float *cm_intra,
                                   const quota_score_params *p, float *score,
                                   float *normed_opt, void *ws, void *stream);

/* Deterministic TopK (Eq. 9): the min(K, Nv) largest scores of each sequence,
 * ties broken towards the lower index, emitted in ascending index order.
 * score fp32 [B][Nv]; keep_idx int32 [B][min(K,Nv)].  K is the integer budget
 * K_l = ceil(r_l * V0) (Eq. 5) -- the rounding is the recipe's job.  NaN
 * scores rank lowest.  Requires Nv <= 8192, K >= 0. */
int quota_topk_prune(const float *score, int B, int Nv, int K,
                     int32_t *keep_idx, void *stream);

/* ---- the whole layer ---------------------------------------------------- */

typedef struct quota_layer {
    int H, dh, F;                /* d = H*dh (H query heads)                  */
    float eps;
    const float *gamma1, *gamma2; /* fp32 [d]                                 */
    quota_weights qkv;           /* [d + 2*Hkv*dh][d], rows q | k | v         */
    quota_weights o;             /* [d][d]                                    */
    quota_weights gu;            /* [2F][d], rows gate | up                   */
    quota_weights down;          /* [d][F]                                    */
    const float *cosT, *sinT;    /* fp32 [n_pos][dh/2]                        */
    int n_pos;
    int Hkv;                     /* K/V heads (grouped-query attention: query
                                  * head h reads K/V head h / (H/Hkv), the cues
                                  * still average over the H query heads);
                                  * 0 = H.  The layer's KV cache then has
                                  * cache->H == Hkv.  Needs H % Hkv == 0.     */
} quota_layer;

/* Layer state (host struct, device buffers).  On entry x holds B sequences of
 * N = vis_begin + Nv + Nt_after rows each (visual tokens in rows
 * [vis_begin, vis_begin+Nv)), pos their original position ids.  On return
 * x_out / pos_out hold the compacted sequences (kept visual tokens + every
 * text token, original order) and N, Nv are updated. */
typedef struct quota_state {
    int B, N, vis_begin, Nv;
    const void *x;       /* fp16 [B][N][d]                                    */
    const int32_t *pos;  /* int32 [B][N]                                      */
    void *x_out;         /* fp16 [B][n_keep][d]                               */
    int32_t *pos_out;    /* int32 [B][n_keep]                                 */
} quota_state;

/* Optional dump / inject points for the parity harness.  Every pointer may be
 * null.  Dumps receive the tensor the layer computed; injects replace it
 * before the next step consumes it. */
typedef struct quota_taps {
    void *qkv;            /* fp16 [B*N][3d]                                   */
    void *q_rot;          /* fp16 [B*N][d]                                    */
    void *o;              /* fp16 [B*N][d] attention output                   */
    float *sumsq, *ressq; /* [B][Nv]                                          */
    float *cm_inter, *cm_intra, *score; /* [B][Nv]                            */
    int32_t *keep_idx;    /* [B][min(K,Nv)]                                   */
    int32_t *rows;        /* [B][n_keep] kept row ids                         */
    void *x1;             /* fp16 [B*n_keep][d]                               */
    void *gu;             /* fp16 [B*n_keep][2F]                              */
    void *z;              /* fp16 [B*n_keep][F]                               */
    const void *inject_o;        /* fp16 [B*N][d]                             */
    const float *inject_cm_inter, *inject_cm_intra; /* [B][Nv]                */
    const void *inject_z;        /* fp16 [B*n_keep][F]                        */
} quota_taps;

size_t quota_prefill_workspace_bytes(const quota_layer *L, int B, int N);

/* K_l value for a layer that is not a pruning candidate (the recipe prunes at
 * the candidate layers only): no cue pass, no score, no top-k; every token is
 * kept. */
#define QUOTA_KEEP_ALL (-1)

/* One decoder layer of the deployed low-bit forward pass (Method overview;
 * Eq. 5-9 and the compaction paragraph): RMSNorm + int4 activations + W4A4
 * QKV, RoPE, 4-bit K/V for all N tokens, causal attention over the 4-bit
 * K/V, the four cues, G, score fusion, top-K_l over the visual tokens, then
 * compaction: kept rows of the hidden state and positions move on, their 4-bit
 * K/V rows are appended to `cache` (this layer's cache), and the output
 * projection and SwiGLU FFN (all token-wise) run on the kept rows only.
 * K_l >= Nv keeps every token but still scores them; K_l = QUOTA_KEEP_ALL marks
 * a layer outside the candidate set: the cue pass, the score and the top-k are
 * skipped.  ws: quota_prefill_workspace_bytes bytes.
 * Every limit of the steps is checked before the first launch, and the
 * descriptors (cache->len, st->N, st->Nv) move only after the last one, so a
 * call that returns an error has enqueued nothing and changed nothing:
 * QUOTA_ERR_SHAPE for dh not 64 / 128, H % Hkv != 0, F % 32 != 0, d > 16384,
 * F > 32768, more than 8192 visual tokens in a candidate layer, weight shapes
 * that do not fit the layer or the packer; QUOTA_ERR_CAPACITY when the cache
 * cannot take n_keep more rows. */
int quota_prefill_layer(const quota_layer *L, quota_state *st, int K_l,
                        const quota_score_params *p, quota_kv_cache *cache,
                        const quota_taps *taps_opt, void *ws, void *stream);

/* ---- offline budget allocation (Eq. 1-5; host arithmetic, HOST pointers) -- */

/* Eq. 1 for one layer: S = median over the n calibration samples of
 * diff_norm[i] / (ref_norm[i] + eta), with diff_norm = ||x^q - x||_2 and
 * ref_norm = ||x||_2 measured by the caller (even n: mean of the two middle
 * values).  QUOTA_ERR_INVALID_ARG for n <= 0, negative inputs or eta, or a
 * zero denominator. */
int quota_sensitivity(const double *diff_norm, const double *ref_norm, int n,
                      double eta, double *S_out);

/* Eq. 2-5: from the raw sensitivities S[m] of the ordered candidate layers to
 * the deployable recipe.  S~ = clip((S - P10)/(P90 - P10), 0.1, 0.9) with
 * linearly interpolated percentiles over the m values (0.5 for all when
 * P90 == P10); pi = softmax((1 - S~)/tau); d_i = (1 - p_min) pi_i;
 * r_i = max(p_min, 1 - sum_{j<=i} d_j); K_i = ceil(r_i V0 - 1e-9).
 * r_out[m], K_out[m] required; s_norm_opt[m], pi_opt[m] optional.  The K_i are
 * what quota_prefill_layer takes as K_l for candidate layer i.
 * Requires m > 0, tau > 0, 0 <= p_min <= 1, V0 >= 0, finite S. */
int quota_make_recipe(const double *S, int m, double tau, double p_min, int V0,
                      double *s_norm_opt, double *pi_opt, double *r_out,
                      int32_t *K_out);

/* GFLOPs ratio (percent) of a pruning recipe against the unpruned model
 * (GFLOPs-estimation appendix): (F_vt + F_pj + sum_l C(T + V_hat[l])) /
 * (F_vt + F_pj + L C(T + V0)), with the per-layer cost of a LLaMA-style block
 * C(S) = 2 S (4 d^2 + 3 d F) + 4 S^2 d (the appendix names the projection/MLP
 * and attention terms but prints no formula; this is the usual count, 2 FLOPs
 * per multiply-add, attention in full).  V_hat[L] (host) = visual tokens
 * executed by each layer; T = text-length proxy. */
int quota_gflops_ratio(const int32_t *V_hat, int L, int V0, int T, int d, int F,
                       double F_vt, double F_pj, double *ratio_percent);

/* ---- sensitivity profiling for Eq. 1 (calibration time; DEVICE pointers) ---- */

/* The full-precision counterpart of quota_layer: the same decoder block with
 * fp16 weights, row-major [N_out][K], same row orders (q | k | v, gate | up),
 * and no quantizer anywhere.  Hkv = 0 means H. */
typedef struct quota_fp_layer {
    int H, dh, F, Hkv;
    float eps;
    const float *gamma1, *gamma2;   /* fp32 [d]                               */
    const void *wqkv;               /* fp16 [d + 2*Hkv*dh][d]                 */
    const void *wo;                 /* fp16 [d][d]                            */
    const void *wgu;                /* fp16 [2F][d]                           */
    const void *wdown;              /* fp16 [d][F]                            */
    const float *cosT, *sinT;       /* fp32 [n_pos][dh/2]                     */
    int n_pos;
} quota_fp_layer;

size_t quota_fp_block_workspace_bytes(const quota_fp_layer *L, int B, int N);

/* The full-precision activation x_l of Eq. 1: one decoder block (RMSNorm,
 * q|k|v projection, rotate-half RoPE at pos, causal softmax attention with
 * grouped K/V heads, output projection + residual, RMSNorm, SwiGLU, +
 * residual) on x fp16 [B][N][d], fp16 storage between the steps, fp32
 * accumulation, nothing quantized.  x_out fp16 [B][N][d].  Calibration-time
 * code, not tuned.  ws: quota_fp_block_workspace_bytes bytes.
 * QUOTA_ERR_SHAPE for dh not 64 / 128, H % Hkv != 0, F % 32 != 0. */
int quota_fp_block(const quota_fp_layer *L, const void *x_f16, const int32_t *pos,
                   int B, int N, void *x_out_f16, void *ws, void *stream);

/* Numerator and denominator of Eq. 1 for each of B samples: diff_norm[b] =
 * ||x^q_b - x_b||_2, ref_norm[b] = ||x_b||_2 over the n_per_sample fp16 values
 * of sample b (all its tokens and channels), accumulated in fp64.  xq, x fp16
 * [B][n_per_sample]; diff_norm, ref_norm fp64 [B] (device).  Copy them to the
 * host for quota_sensitivity. */
int quota_activation_deviation(const void *xq_f16, const void *x_f16, int B,
                               long n_per_sample, double *diff_norm,
                               double *ref_norm, void *stream);

size_t quota_profile_block_workspace_bytes(const quota_layer *Lq, const quota_fp_layer *Lf,
                                           int B, int N);

/* Eq. 1's measurement for one block and B calibration samples: runs the
 * deployed low-bit block (quota_prefill_layer with QUOTA_KEEP_ALL: calibration
 * precedes the recipe, nothing is pruned) and the full-precision block on the
 * same input x / pos, and returns the per-sample norms of the difference and
 * of the full-precision output (device fp64 [B]).  Both runs start from the
 * same block input, so the deviation is this block's own.  scratch_cache: a
 * cache descriptor of this layer's geometry with room for N more rows; its
 * rows beyond len are overwritten and len is left as it came.
 * ws: quota_profile_block_workspace_bytes bytes.  Errors as the two block
 * calls; QUOTA_ERR_SHAPE when the two layers' geometries differ. */
int quota_profile_block(const quota_layer *Lq, const quota_fp_layer *Lf,
                        const void *x_f16, const int32_t *pos, int B, int N,
                        quota_kv_cache *scratch_cache, double *diff_norm,
                        double *ref_norm, void *ws, void *stream);

/* ---- decode over the pruned 4-bit KV cache ------------------------------- */

/* Single-query attention of one new token per sequence over `cache` (deployment
 * pipeline: decoding reads the quantized KV cache that holds retained tokens
 * only).  q fp16 [B][H*dh] (rotated); rows 0..len-1 of every sequence are read
 * -- the new token's own K/V must already be appended -- as
 * x_hat = fp16(code * scale); scores q.k_hat/sqrt(dh), fp32 softmax,
 * o fp16 [B][H*dh].  B, H, dh, len come from the cache descriptor.
 * Requires dh == 64 or 128 and 1 <= len <= 8192 (QUOTA_ERR_SHAPE beyond). */
int quota_attention_decode(const void *q_f16, const quota_kv_cache *cache,
                           void *o_f16, void *stream);

/* The same for grouped-query attention: q and o have Hq heads per row, the
 * cache holds cache->H K/V heads, query head h reads K/V head h / (Hq/cache->H).
 * Requires Hq % cache->H == 0. */
int quota_attention_decode_gqa(const void *q_f16, int Hq, const quota_kv_cache *cache,
                               void *o_f16, void *stream);

/* *step_dev += 1 on the stream (a one-thread kernel, so it can be captured in
 * the same HIP graph as the decode step that reads it). */
int quota_advance_step(int32_t *step_dev, void *stream);

size_t quota_decode_workspace_bytes(const quota_layer *L, int B);

/* One decode step of one layer for one new token per sequence: RMSNorm +
 * quantizer + W4A4 QKV, RoPE at the token's original position id pos[b], 4-bit
 * quantization of its K/V exactly as for prefill rows, append at row
 * cache->len (advanced by 1), attention over the whole cache, then the
 * token-wise output projection and SwiGLU FFN.  Nothing is pruned at decode.
 * x fp16 [B][d], pos int32 [B], x_out fp16 [B][d] (all device); B must equal
 * cache->B.  taps_opt: qkv, q_rot, o, x1, gu, z dumps and inject_o / inject_z
 * are honoured (parity harness).  ws: quota_decode_workspace_bytes bytes.
 * Checked before the first launch: QUOTA_ERR_CAPACITY when the cache is full,
 * QUOTA_ERR_SHAPE when it would hold more than 8192 rows or for the layer
 * shapes quota_prefill_layer rejects; cache->len is advanced after the last
 * launch, so an error leaves the cache as it was. */
int quota_decode_layer(const quota_layer *L, const void *x_f16,
                       const int32_t *pos, int B, quota_kv_cache *cache,
                       void *x_out_f16, const quota_taps *taps_opt, void *ws,
                       void *stream);

/* ---- per-kernel timing for benchmarks ----------------------------------- */

/* Kernel classes the library launches.  The GEMM is split by tile shape
 * because each shape is a separate kernel (and a separate profiler row). */
enum {
    QUOTA_K_QUANTIZE_ACT = 0, QUOTA_K_RMSNORM_QUANTIZE_ACT, QUOTA_K_SILU_MUL_QUANTIZE_ACT,
    QUOTA_K_GEMM_64X256, QUOTA_K_GEMM_64X128, QUOTA_K_GEMM_32X128, QUOTA_K_GEMM_32X128_DEEP, QUOTA_K_GEMM_64X128_LEAN,
    QUOTA_K_GEMM_OTHER, QUOTA_K_ROPE_KV_QUANT,
    QUOTA_K_KV_QUANT_APPEND, QUOTA_K_ATTENTION_FWD, QUOTA_K_ATTENTION_COLMASS,
    QUOTA_K_SCORE_TOKENS, QUOTA_K_TOPK_PRUNE, QUOTA_K_COMPACT_ROWS, QUOTA_K_QUANTIZE_WEIGHTS,
    QUOTA_K_PACK_WEIGHTS, QUOTA_K_ATTENTION_DECODE, QUOTA_K_KV_APPEND_ROWS, QUOTA_K_GEMM_ROWS16, QUOTA_KERNEL_COUNT
};

/* Per kernel class: launches seen, summed HIP-event time around them (ms) and
 * the ALGORITHMIC work those launches stood for: integer/float operations
 * (2 per multiply-add) and bytes the operation must move (inputs read once +
 * outputs written once, int4 data counted as half bytes). */
typedef struct quota_kernel_stat {
    long launches;
    double total_ms;
    double ops;
    double bytes;
} quota_kernel_stat;

const char *quota_kernel_name(int kernel_id);

/* Starts recording a HIP-event pair around every kernel launch the library
 * makes (on the launch's own stream), for at most max_launches launches; more
 * are not recorded.  Allocates host memory and HIP events: not for the hot
 * path, and recording must not be active during HIP graph capture. */
int quota_profile_begin(int max_launches);

/* Stops recording, waits for the recorded events, fills
 * stats[QUOTA_KERNEL_COUNT] (host) and frees the events. */
int quota_profile_collect(quota_kernel_stat *stats);

/* The fixed cost of an event pair itself.  On `stream`, brackets one empty
 * kernel, then two, between a pair of HIP events, `reps` (1..1024) times each,
 * and takes medians t1 and t2.  t2 - t1 is what one more empty kernel adds
 * (*empty_kernel_ms, optional); t1 - (t2 - t1) is what the bracket costs with
 * no kernel in it (*bracket_ms) -- the part of quota_profile_collect's
 * total_ms, per launch, that is not the kernel's.  Both are host pointers.
 * Allocates events: benchmark use only. */
int quota_profile_bracket_ms(int reps, void *stream, float *bracket_ms, float *empty_kernel_ms);

#ifdef __cplusplus
}
#endif
#endif /* QUOTA_H */
