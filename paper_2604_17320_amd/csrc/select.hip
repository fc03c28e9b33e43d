// Token scoring (Eq. 6-8) and deterministic budgeted top-k (Eq. 9).
// One workgroup per sequence.  Order statistics and the top-k threshold come
// from an exact 4-pass, 8-bit radix select on order-preserving uint32 keys,
// run by ONE WAVE with a private 256-bin LDS histogram (integer atomics, so
// the result does not depend on execution order; no workgroup barrier inside
// the select).  The eight percentile bounds of the four metrics are found in
// parallel, one wave each; the top-k runs on wave 0.
#include "common.h"
#include "internal.h"

namespace {

constexpr int MAXV = QUOTA_MAX_SCORED_TOKENS;

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

// Inclusive prefix sum over the 64 lanes of a wave with DPP moves (no LDS crossbar): shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then lane 15 of rows 0 and 2 is added to rows 1 and 3,
// then lane 31 to rows 2 and 3.  Lanes without a source add 0.
__device__ __forceinline__ int wave_incl_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);     // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);     // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);     // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);     // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);     // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);     // row_bcast:31 -> rows 2, 3
    return v;
}

// Exact k-th smallest (0-based rank) of the n keys key_at(i), computed by the
// calling wave alone.  hist: 256 ints of LDS private to the wave.  All lanes
// return the key.
template <typename KeyAt>
__device__ uint32_t wave_radix_select(KeyAt key_at, int n, int rank, volatile int *hist)
{
    const int lane = threadIdx.x & 63;
    uint32_t prefix = 0, mask = 0;
    int remaining = rank;
    for (int shift = 24; shift >= 0; shift -= 8) {
#pragma unroll
        for (int b = 0; b < 4; ++b) hist[4 * lane + b] = 0;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        for (int i = lane; i < n; i += 64) {
            uint32_t k = key_at(i);
            if ((k & mask) == prefix) atomicAdd(const_cast<int *>(&hist[(k >> shift) & 0xFF]), 1);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        int c0 = hist[4 * lane], c1 = hist[4 * lane + 1], c2 = hist[4 * lane + 2], c3 = hist[4 * lane + 3];
        const int s = c0 + c1 + c2 + c3, incl = wave_incl_scan(s);
        int excl = incl - s;
        bool mine = remaining >= excl && remaining < incl;      // exactly one lane
        int r = remaining - excl, digit = 4 * lane;
        if (r >= c0) { r -= c0; ++digit;
            if (r >= c1) { r -= c1; ++digit;
                if (r >= c2) { r -= c2; ++digit; } } }
        unsigned long long who = __ballot(mine);
        int src = __ffsll((long long)who) - 1;
        digit = __shfl(digit, src, 64);
        remaining = __shfl(r, src, 64);
        prefix |= (uint32_t)digit << shift;
        mask |= 0xFFu << shift;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
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

struct MetricSrc {
    const float *sumsq, *ressq, *cm_inter, *cm_intra;
    const float *partial;   // optional per-head column masses [B][H][Nv][2] (text, visual)
    int H;
    float *cm_out_inter, *cm_out_intra;     // optional [B][Nv] outputs of the head means
    size_t osq, ocm;        // offsets of this sequence in the sumsq/ressq and cm arrays
};

constexpr int SCORE_THREADS = 1024;

// Loads the four Eq. 6 metrics of sequence b into LDS as order-preserving keys, finds the
// eight percentile bounds (one wave per bound, keys in LDS), then fuses the score of every
// token.  1024 threads: the load phase is one memory round trip deep -- a thread owns a
// quarter of the heads of up to three tokens and issues all those loads back to back.
// mk: 4*cap keys (cap >= Nv: the stride between the four metrics), hist: 8*256 ints, lohi: 8 floats.
template <int PER>      // tokens per thread of the fusion pass: Nv <= PER * SCORE_THREADS
__device__ void score_phase(const MetricSrc &src, int B, int Nv, int b, const quota_score_params &p,
                            float *__restrict__ score, float *__restrict__ normed, uint32_t *mk, int cap,
                            int *hist, float *lohi)
{
    const int tid = threadIdx.x, wave = tid >> 6;
    if (src.partial) {
        // head mean: lane quarter hq sums heads [hq*H/4 .. ) in head order, the four partial
        // sums are combined as (s0 + s1) + (s2 + s3), then * (1/H)
        const int hq = tid & 3, hper = (src.H + 3) / 4, h_lo = hq * hper, h_hi = min(h_lo + hper, src.H);
        const float2 *pp = reinterpret_cast<const float2 *>(src.partial) + (size_t)b * src.H * Nv;
        const float invH = 1.0f / (float)src.H;
        for (int i0 = 0; i0 < Nv; i0 += 3 * (SCORE_THREADS / 4)) {
            float st[3] = {0.0f, 0.0f, 0.0f}, sv[3] = {0.0f, 0.0f, 0.0f};
            for (int h0 = h_lo; h0 < h_hi; h0 += 8) {
                float2 v[3][8];
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const int i = i0 + (tid >> 2) + r * (SCORE_THREADS / 4);
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        v[r][u] = (i < Nv && h0 + u < h_hi) ? pp[(size_t)(h0 + u) * Nv + i] : make_float2(0.0f, 0.0f);
                }
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int u = 0; u < 8; ++u) { st[r] += v[r][u].x; sv[r] += v[r][u].y; }
            }
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const int i = i0 + (tid >> 2) + r * (SCORE_THREADS / 4);
                float a = st[r], c = sv[r];
                a += __shfl_xor(a, 1, 64); c += __shfl_xor(c, 1, 64);
                a += __shfl_xor(a, 2, 64); c += __shfl_xor(c, 2, 64);
                if (i < Nv && hq == 0) {
                    const float m_inter = a * invH, m_intra = c * invH;
                    if (src.cm_out_inter) src.cm_out_inter[src.ocm + i] = m_inter;
                    if (src.cm_out_intra) src.cm_out_intra[src.ocm + i] = m_intra;
                    mk[1 * cap + i] = float_key(m_inter);
                    mk[2 * cap + i] = float_key(m_intra);
                }
            }
        }
    }
    for (int i = tid; i < Nv; i += SCORE_THREADS) {
        if (!src.partial) {
            mk[1 * cap + i] = float_key(src.cm_inter[src.ocm + i]);
            mk[2 * cap + i] = float_key(src.cm_intra[src.ocm + i]);
        }
        mk[0 * cap + i] = float_key(sqrtf(src.sumsq[src.osq + i]));    // m_mag
        mk[3 * cap + i] = float_key(sqrtf(src.ressq[src.osq + i]));    // m_res
    }
    __syncthreads();
    const int r_lo = (p.pct_lo * (Nv - 1) + 50) / 100, r_hi = (p.pct_hi * (Nv - 1) + 50) / 100;
    if (wave < 8) {                                 // wave 2m: low bound of metric m, wave 2m+1: high bound
        const uint32_t *keys = mk + (wave >> 1) * cap;
        auto key_at = [&](int i) { return keys[i]; };
        uint32_t kb = wave_radix_select(key_at, Nv, (wave & 1) ? r_hi : r_lo, hist + 256 * wave);
        if ((tid & 63) == 0) lohi[wave] = key_float(kb);
    }
    __syncthreads();
    float sc[PER];
#pragma unroll
    for (int r = 0; r < PER; ++r) {
        const int i = tid + SCORE_THREADS * r;
        if (i < Nv) {
            float g0 = robust_unit(key_float(mk[0 * cap + i]), lohi[0], lohi[1]);
            float g1 = robust_unit(key_float(mk[1 * cap + i]), lohi[2], lohi[3]);
            float g2 = robust_unit(key_float(mk[2 * cap + i]), lohi[4], lohi[5]);
            float g3 = robust_unit(key_float(mk[3 * cap + i]), lohi[6], lohi[7]);
            float a = p.w_m * g0;
            float c = p.w_c * g1;
            float s = p.w_s * g2;
            float rr = p.w_r * g3;
            float acc = a + c;
            acc = acc + s;
            acc = acc + rr;
            size_t o = (size_t)b * Nv + i;
            score[o] = acc;
            sc[r] = acc;
            if (normed) {
                size_t plane = (size_t)B * Nv;
                normed[0 * plane + o] = g0;
                normed[1 * plane + o] = g1;
                normed[2 * plane + o] = g2;
                normed[3 * plane + o] = g3;
            }
        }
    }
    __syncthreads();            // every metric key has been read: slot 0 becomes the score keys
#pragma unroll
    for (int r = 0; r < PER; ++r) {
        const int i = tid + SCORE_THREADS * r;
        if (i < Nv) mk[i] = (sc[r] != sc[r]) ? 0u : float_key(sc[r]);
    }
}

__device__ __forceinline__ int wave_excl_scan(int v, int *total)
{
    const int incl = wave_incl_scan(v);
    *total = __shfl(incl, 63, 64);
    return incl - v;
}

// Top-k of keys[0..Nv) (LDS) by the calling wave: K largest, ties to the lower
// index, ascending output.  Requires 0 < K < Nv.
__device__ void topk_phase(const uint32_t *keys, int Nv, int K, int32_t *__restrict__ out, int *hist)
{
    const int lane = threadIdx.x & 63;
    auto key_at = [&](int i) { return keys[i]; };
    // threshold = K-th largest = rank (Nv - K) in ascending order
    const uint32_t thr = wave_radix_select(key_at, Nv, Nv - K, hist);
    // each lane owns a contiguous index range so the scans follow index order
    const int per = (Nv + 63) / 64;
    const int i0 = min(lane * per, Nv), i1 = min(i0 + per, Nv);
    int n_gt = 0, n_eq = 0;
    for (int i = i0; i < i1; ++i) {
        n_gt += keys[i] > thr;
        n_eq += keys[i] == thr;
    }
    int tot_gt, tot_eq;
    const int eq_before = wave_excl_scan(n_eq, &tot_eq);
    wave_excl_scan(n_gt, &tot_gt);
    const int need = K - tot_gt;                       // ties taken, lowest indices first
    int n_sel = 0, e = eq_before;
    for (int i = i0; i < i1; ++i) {
        uint32_t k = keys[i];
        n_sel += (k > thr) || (k == thr && e < need);
        e += k == thr;
    }
    int tot_sel;
    int pos = wave_excl_scan(n_sel, &tot_sel);
    e = eq_before;
    for (int i = i0; i < i1; ++i) {
        uint32_t k = keys[i];
        if ((k > thr) || (k == thr && e < need)) out[pos++] = i;
        e += k == thr;
    }
}

// K < 0: score only.  When K >= 0 the indices of the min(K, Nv) best tokens of
// sequence b go to keep_idx[b][0..min(K,Nv)).
template <int PER>
__global__ __launch_bounds__(SCORE_THREADS) void score_topk_kernel(MetricSrc src, long stride_sq, int B, int Nv,
                                                         quota_score_params p,
                                                         float *__restrict__ score,
                                                         float *__restrict__ normed, int K,
                                                         int32_t *__restrict__ keep_idx, int cap)
{
    // LDS sized by the launch for this Nv: 4 * cap keys, 8 histograms of 256 bins, 8 bounds
    extern __shared__ __align__(16) uint32_t score_lds[];
    uint32_t *mk = score_lds;
    int *hist = reinterpret_cast<int *>(mk + 4 * cap);
    float *lohi = reinterpret_cast<float *>(hist + 8 * 256);
    const int b = blockIdx.x;
    src.osq = (size_t)b * stride_sq;
    src.ocm = (size_t)b * Nv;
    score_phase<PER>(src, B, Nv, b, p, score, normed, mk, cap, hist, lohi);
    if (K < 0) return;
    const int k = K < Nv ? K : Nv;
    int32_t *out = keep_idx + (size_t)b * k;
    if (k == Nv) {
        for (int i = threadIdx.x; i < Nv; i += SCORE_THREADS) out[i] = i;
        return;
    }
    __syncthreads();
    if (threadIdx.x < 64 && k > 0) topk_phase(mk, Nv, k, out, hist);
}

__global__ __launch_bounds__(256) void topk_kernel(const float *__restrict__ score, int Nv, int K,
                                                   int32_t *__restrict__ keep_idx)
{
    __shared__ uint32_t keys[MAXV];
    __shared__ int hist[256];
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
    __syncthreads();
    if (threadIdx.x < 64) topk_phase(keys, Nv, K, out, hist);
}

// Launches the score (+ top-k) kernel with the LDS its Nv needs: up to 136 KB at 8192 tokens, which
// is above the default limit of a launch and has to be granted once per device.
int launch_score_topk(const MetricSrc &src, long stride_sq, int B, int Nv, const quota_score_params &p,
                      float *score, float *normed, int K, int32_t *keep_idx, hipStream_t st)
{
    const int cap = (Nv + 63) & ~63;
    const size_t lds = ((size_t)4 * cap + 8 * 256 + 8) * sizeof(uint32_t);
    if (Nv > 3 * SCORE_THREADS) {          // the widest instantiation: up to 136 KB, above a launch's default 64 KB
        static bool granted[64];
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return QUOTA_ERR_HIP;
        if (!granted[dev]) {
            const size_t most = ((size_t)4 * MAXV + 8 * 256 + 8) * sizeof(uint32_t);
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(score_topk_kernel<MAXV / SCORE_THREADS>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)most) != hipSuccess)
                return QUOTA_ERR_HIP;
            granted[dev] = true;
        }
    }
    auto kernel = Nv <= SCORE_THREADS ? score_topk_kernel<1>
                  : Nv <= 3 * SCORE_THREADS ? score_topk_kernel<3> : score_topk_kernel<MAXV / SCORE_THREADS>;
    kernel<<<dim3(B), dim3(SCORE_THREADS), lds, st>>>(src, stride_sq, B, Nv, p, score, normed, K, keep_idx, cap);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

int check_score_args(const float *sumsq, const float *ressq, const float *cm_inter,
                     const float *cm_intra, int B, int Nv, const quota_score_params *p, float *score)
{
    if (!sumsq || !ressq || !cm_inter || !cm_intra || !p || !score) return QUOTA_ERR_NULL;
    if (B <= 0 || Nv < 0 || p->pct_lo < 0 || p->pct_hi > 100 || p->pct_lo > p->pct_hi)
        return QUOTA_ERR_INVALID_ARG;
    if (Nv > MAXV) return QUOTA_ERR_SHAPE;
    return QUOTA_OK;
}

}  // namespace

int quota_internal_score(const float *sumsq, const float *ressq, long stride_sq,
                         const float *cm_inter, const float *cm_intra, int B, int Nv,
                         const quota_score_params *p, float *score, float *normed, hipStream_t st)
{
    int rc = check_score_args(sumsq, ressq, cm_inter, cm_intra, B, Nv, p, score);
    if (rc != QUOTA_OK) return rc;
    if (Nv == 0) return QUOTA_OK;
    ProfScope prof(QUOTA_K_SCORE_TOKENS, 0, 20.0 * B * Nv, st);
    MetricSrc src{sumsq, ressq, cm_inter, cm_intra, nullptr, 0, nullptr, nullptr, 0, 0};
    return launch_score_topk(src, stride_sq, B, Nv, *p, score, normed, -1, nullptr, st);
}

// score + top-k in one launch (the layer's path).  The attention cues come either as
// head-averaged arrays (cm_inter / cm_intra) or, when `partial` is given, as the
// per-head column masses [B][H][Nv][2] whose head mean is taken here; cm_out_* (optional)
// then receive the head means.
int quota_internal_score_topk(const float *sumsq, const float *ressq, long stride_sq,
                              const float *cm_inter, const float *cm_intra, const float *partial,
                              int H, float *cm_out_inter, float *cm_out_intra, int B, int Nv,
                              const quota_score_params *p, float *score, int K, int32_t *keep_idx,
                              hipStream_t st)
{
    if (!sumsq || !ressq || !p || !score || !keep_idx) return QUOTA_ERR_NULL;
    if (!partial && (!cm_inter || !cm_intra)) return QUOTA_ERR_NULL;
    if (B <= 0 || Nv < 0 || K < 0 || (partial && H <= 0) || p->pct_lo < 0 || p->pct_hi > 100 ||
        p->pct_lo > p->pct_hi)
        return QUOTA_ERR_INVALID_ARG;
    if (Nv > MAXV) return QUOTA_ERR_SHAPE;
    if (Nv == 0) return QUOTA_OK;
    ProfScope prof(QUOTA_K_SCORE_TOKENS, 0,
                   (partial ? 8.0 * H + 8 : 20.0) * B * Nv + 4.0 * B * (K < Nv ? K : Nv), st);
    MetricSrc src{sumsq, ressq, cm_inter, cm_intra, partial, H, cm_out_inter, cm_out_intra, 0, 0};
    return launch_score_topk(src, stride_sq, B, Nv, *p, score, nullptr, K, keep_idx, st);
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
