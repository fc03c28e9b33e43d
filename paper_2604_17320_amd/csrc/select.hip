// Token scoring (Eq. 6-8) and deterministic budgeted top-k (Eq. 9).
// One 256-thread workgroup per sequence; the Nv <= 4096 values live in LDS and
// order statistics / the top-k threshold come from an exact 4-pass, 8-bit
// radix select on order-preserving uint32 keys (LDS integer histograms, so the
// result does not depend on execution order).
#include "common.h"
#include "internal.h"

namespace {

constexpr int MAXV = 4096;

// ascending uint32 order == ascending float order; -0 is folded onto +0
__device__ __forceinline__ uint32_t float_key(float f)
{
    f = f + 0.0f;
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k)
{
    uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __uint_as_float(u);
}

// Exact k-th smallest (0-based rank) of keys[0..n), whole block cooperates.
// hist: 256 ints of LDS; bc: 2 ints of LDS.  All threads return the key.
__device__ uint32_t radix_select(const uint32_t *keys, int n, int rank, int *hist, int *bc)
{
    uint32_t prefix = 0, mask = 0;
    int remaining = rank;
    for (int shift = 24; shift >= 0; shift -= 8) {
        __syncthreads();
        hist[threadIdx.x] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < n; i += 256) {
            uint32_t k = keys[i];
            if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 0xFF], 1);
        }
        __syncthreads();
        if (threadIdx.x < 64) {          // wave 0 scans the 256 bins, 4 per lane
            int l = threadIdx.x;
            int c0 = hist[4 * l], c1 = hist[4 * l + 1], c2 = hist[4 * l + 2], c3 = hist[4 * l + 3];
            int s = c0 + c1 + c2 + c3, incl = s;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                int t = __shfl_up(incl, off, 64);
                if (l >= off) incl += t;
            }
            int excl = incl - s;
            if (remaining >= excl && remaining < incl) {   // exactly one lane
                int r = remaining - excl, digit = 4 * l;
                if (r >= c0) { r -= c0; ++digit;
                    if (r >= c1) { r -= c1; ++digit;
                        if (r >= c2) { r -= c2; ++digit; } } }
                bc[0] = digit;
                bc[1] = r;
            }
        }
        __syncthreads();
        prefix |= (uint32_t)bc[0] << shift;
        mask |= 0xFFu << shift;
        remaining = bc[1];
    }
    __syncthreads();
    return prefix;
}

// G (Eq. 7): clip to the nearest-rank percentiles and rescale to [0, 1]
__device__ __forceinline__ float robust_unit(float m, float lo, float hi)
{
    if (hi == lo) return 0.5f;
    float num = m - lo;
    float den = hi - lo;
    float v = num / den;
    return fminf(fmaxf(v, 0.0f), 1.0f);
}

__device__ __forceinline__ float metric_value(int k, size_t isq, size_t icm,
                                              const float *__restrict__ sumsq,
                                              const float *__restrict__ ressq,
                                              const float *__restrict__ cm_inter,
                                              const float *__restrict__ cm_intra)
{
    switch (k) {
    case 0: return sqrtf(sumsq[isq]);          // m_mag
    case 1: return cm_inter[icm];              // m_inter
    case 2: return cm_intra[icm];              // m_intra
    default: return sqrtf(ressq[isq]);         // m_res
    }
}

__global__ __launch_bounds__(256) void score_kernel(
    const float *__restrict__ sumsq, const float *__restrict__ ressq, long stride_sq,
    const float *__restrict__ cm_inter, const float *__restrict__ cm_intra, int B, int Nv,
    quota_score_params p, float *__restrict__ score, float *__restrict__ normed)
{
    __shared__ uint32_t keys[MAXV];
    __shared__ int hist[256];
    __shared__ int bc[2];
    const int b = blockIdx.x;
    const int r_lo = (p.pct_lo * (Nv - 1) + 50) / 100, r_hi = (p.pct_hi * (Nv - 1) + 50) / 100;
    float lo[4], hi[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        __syncthreads();
        for (int i = threadIdx.x; i < Nv; i += 256)
            keys[i] = float_key(metric_value(k, (size_t)b * stride_sq + i, (size_t)b * Nv + i, sumsq,
                                             ressq, cm_inter, cm_intra));
        lo[k] = key_float(radix_select(keys, Nv, r_lo, hist, bc));
        hi[k] = key_float(radix_select(keys, Nv, r_hi, hist, bc));
    }
    for (int i = threadIdx.x; i < Nv; i += 256) {
        size_t isq = (size_t)b * stride_sq + i, icm = (size_t)b * Nv + i;
        float g0 = robust_unit(metric_value(0, isq, icm, sumsq, ressq, cm_inter, cm_intra), lo[0], hi[0]);
        float g1 = robust_unit(metric_value(1, isq, icm, sumsq, ressq, cm_inter, cm_intra), lo[1], hi[1]);
        float g2 = robust_unit(metric_value(2, isq, icm, sumsq, ressq, cm_inter, cm_intra), lo[2], hi[2]);
        float g3 = robust_unit(metric_value(3, isq, icm, sumsq, ressq, cm_inter, cm_intra), lo[3], hi[3]);
        float a = p.w_m * g0;
        float c = p.w_c * g1;
        float s = p.w_s * g2;
        float r = p.w_r * g3;
        float acc = a + c;
        acc = acc + s;
        acc = acc + r;
        score[icm] = acc;
        if (normed) {
            size_t plane = (size_t)B * Nv;
            normed[0 * plane + icm] = g0;
            normed[1 * plane + icm] = g1;
            normed[2 * plane + icm] = g2;
            normed[3 * plane + icm] = g3;
        }
    }
}

// block-wide exclusive scan of one int per thread (256 threads)
__device__ __forceinline__ int block_excl_scan(int v, int *sm, int *total)
{
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
    }
    __syncthreads();
    if (lane == 63) sm[w] = incl;
    __syncthreads();
    int base = 0;
    for (int i = 0; i < w; ++i) base += sm[i];
    *total = sm[0] + sm[1] + sm[2] + sm[3];
    return base + incl - v;
}

__global__ __launch_bounds__(256) void topk_kernel(const float *__restrict__ score, int Nv, int K,
                                                   int32_t *__restrict__ keep_idx)
{
    __shared__ uint32_t keys[MAXV];
    __shared__ int hist[256];
    __shared__ int bc[2];
    __shared__ int sc[4];
    const int b = blockIdx.x;
    int32_t *out = keep_idx + (size_t)b * K;
    if (K >= Nv) {          // host passes K <= Nv; K == Nv keeps every token
        for (int i = threadIdx.x; i < Nv; i += 256) out[i] = i;
        return;
    }
    for (int i = threadIdx.x; i < Nv; i += 256) {
        float f = score[(size_t)b * Nv + i];
        keys[i] = (f != f) ? 0u : float_key(f);       // NaN ranks lowest
    }
    // threshold = K-th largest = rank (Nv - K) in ascending order
    const uint32_t thr = radix_select(keys, Nv, Nv - K, hist, bc);
    // each thread owns a contiguous index range so scans follow index order
    const int per = (Nv + 255) / 256;
    const int i0 = threadIdx.x * per, i1 = min(i0 + per, Nv);
    int n_gt = 0, n_eq = 0;
    for (int i = i0; i < i1; ++i) {
        n_gt += keys[i] > thr;
        n_eq += keys[i] == thr;
    }
    int tot_gt, tot_eq;
    int eq_before = block_excl_scan(n_eq, sc, &tot_eq);
    block_excl_scan(n_gt, sc, &tot_gt);
    const int need = K - tot_gt;                       // ties taken, lowest indices first
    int n_sel = 0, e = eq_before;
    for (int i = i0; i < i1; ++i) {
        uint32_t k = keys[i];
        n_sel += (k > thr) || (k == thr && e < need);
        e += k == thr;
    }
    int tot_sel;
    int pos = block_excl_scan(n_sel, sc, &tot_sel);
    e = eq_before;
    for (int i = i0; i < i1; ++i) {
        uint32_t k = keys[i];
        if ((k > thr) || (k == thr && e < need)) out[pos++] = i;
        e += k == thr;
    }
}

}  // namespace

int quota_internal_score(const float *sumsq, const float *ressq, long stride_sq,
                         const float *cm_inter, const float *cm_intra, int B, int Nv,
                         const quota_score_params *p, float *score, float *normed, hipStream_t st)
{
    if (!sumsq || !ressq || !cm_inter || !cm_intra || !p || !score) return QUOTA_ERR_NULL;
    if (B <= 0 || Nv < 0 || p->pct_lo < 0 || p->pct_hi > 100 || p->pct_lo > p->pct_hi)
        return QUOTA_ERR_INVALID_ARG;
    if (Nv > MAXV) return QUOTA_ERR_SHAPE;
    if (Nv == 0) return QUOTA_OK;
    ProfScope prof(QUOTA_K_SCORE_TOKENS, 0, 20.0 * B * Nv, st);
    score_kernel<<<dim3(B), dim3(256), 0, st>>>(sumsq, ressq, stride_sq, cm_inter, cm_intra, B, Nv,
                                                *p, score, normed);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" void quota_score_params_default(quota_score_params *p)
{
    if (!p) return;
    p->w_m = 0.25f; p->w_c = 0.45f; p->w_s = 0.10f; p->w_r = 0.20f;
    p->pct_lo = 10; p->pct_hi = 90;
}

extern "C" int quota_score_tokens(const float *sumsq, const float *ressq, const float *cm_inter,
                                  const float *cm_intra, int B, int Nv,
                                  const quota_score_params *p, float *score, float *normed_opt,
                                  void *stream)
{
    return quota_internal_score(sumsq, ressq, Nv, cm_inter, cm_intra, B, Nv, p, score, normed_opt,
                                (hipStream_t)stream);
}

extern "C" int quota_topk_prune(const float *score, int B, int Nv, int K, int32_t *keep_idx,
                                void *stream)
{
    if (!score || !keep_idx) return QUOTA_ERR_NULL;
    if (B <= 0 || Nv < 0 || K < 0) return QUOTA_ERR_INVALID_ARG;
    if (Nv > MAXV) return QUOTA_ERR_SHAPE;
    int k = K < Nv ? K : Nv;
    if (k == 0) return QUOTA_OK;
    ProfScope prof(QUOTA_K_TOPK_PRUNE, 0, 4.0 * B * Nv + 4.0 * B * k, (hipStream_t)stream);
    topk_kernel<<<dim3(B), dim3(256), 0, (hipStream_t)stream>>>(score, Nv, k, keep_idx);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" int quota_score_tokens_from_hidden(const void *v_f16, int B, int Nv, int d, int ldv,
                                              long stride_b, const float *cm_inter,
                                              const float *cm_intra, const quota_score_params *p,
                                              float *score, float *normed_opt, void *ws,
                                              void *stream)
{
    if (!ws) return QUOTA_ERR_NULL;
    if (B <= 0 || Nv < 0) return QUOTA_ERR_INVALID_ARG;
    float *sumsq = (float *)ws, *ressq = sumsq + (size_t)B * Nv;
    int rc = quota_internal_vector_metrics(v_f16, B, Nv, d, ldv, stride_b, sumsq, ressq,
                                           (hipStream_t)stream);
    if (rc != QUOTA_OK) return rc;
    return quota_internal_score(sumsq, ressq, Nv, cm_inter, cm_intra, B, Nv, p, score, normed_opt,
                                (hipStream_t)stream);
}

extern "C" const char *quota_strerror(int code)
{
    switch (code) {
    case QUOTA_OK: return "ok";
    case QUOTA_ERR_NULL: return "a required pointer is null";
    case QUOTA_ERR_INVALID_ARG: return "invalid argument";
    case QUOTA_ERR_SHAPE: return "shape not supported by the kernels";
    case QUOTA_ERR_CAPACITY: return "KV cache or workspace capacity exceeded";
    case QUOTA_ERR_HIP: return "HIP runtime reported a launch error";
    default: return "unknown error code";
    }
}

extern "C" int quota_version(void) { return 100; }
