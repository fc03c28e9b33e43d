/*
 * CPU oracle for the QUOTA hot path (W4A4 prefill layer with in-layer visual
 * token pruning and a 4-bit KV cache).
 *
 * THIS IS TEST INFRASTRUCTURE, not the product.  It is a plain, slow, step by
 * step implementation of what the method computes, written from the paper's
 * definitions (Method section: unified low-bit execution form, Eq. 5 budget,
 * Eq. 6 metrics, Eq. 7 robust normalisation, Eq. 8 score fusion, Eq. 9 top-k,
 * and the compaction paragraph that follows Eq. 9).  It shares no code, no
 * header, no table and no helper with the HIP library.  Only tests, the smoke
 * check and the benchmark's CPU-baseline leg may call it.
 *
 * Conventions
 *   - fp16 tensors travel as uint16_t bit patterns (IEEE binary16).
 *   - int4 codes travel unpacked, one int8_t in [-8, 7] per element.
 *   - every tensor that leaves a step is rounded to its storage type there
 *     (fp16 round-to-nearest-even for activations, fp32 for scales/metrics).
 *   - reductions that feed a rounding decision later on (sums of squares, the
 *     attention sums) are accumulated in fp64; elementwise arithmetic that
 *     decides an int4 code is done in fp32 with one IEEE operation per step,
 *     so the file must be compiled with -ffp-contract=off.
 *   - OpenMP "parallel for" over independent rows only.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * against closed forms, invariants, brute force or library routines, except
 * where a header comment says "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ fp16 */

/* binary16 bits -> float (exact). */
static float h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t m = h & 0x3FFu;
    uint32_t bits;
    if (e == 0) {
        if (m == 0) {
            bits = sign;
        } else {            /* subnormal: value = m * 2^-24 */
            float v = (float)m * 5.9604644775390625e-08f;
            memcpy(&bits, &v, 4);
            bits |= sign;
        }
    } else if (e == 31) {
        bits = sign | 0x7F800000u | (m << 13);
    } else {
        bits = sign | ((e + 112u) << 23) | (m << 13);
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* double -> binary16 bits, round to nearest even, one rounding.  Because
 * float -> double is exact this is also the float -> binary16 rounding. */
static uint16_t d2h(double x)
{
    uint16_t sign = 0;
    if (x != x) return 0x7E00u;
    if (signbit(x)) { sign = 0x8000u; x = -x; }
    if (x == 0.0) return sign;
    if (x >= 65520.0) return sign | 0x7C00u;          /* rounds to inf */
    int ex;
    (void)frexp(x, &ex);                              /* x = f * 2^ex, f in [0.5,1) */
    int e = ex - 1;                                   /* x = 1.f * 2^e            */
    if (e < -14) e = -14;                             /* subnormal spacing 2^-24  */
    /* spacing of representable values in this binade is 2^(e-10) */
    double scaled = ldexp(x, 10 - e);                 /* in [0, 2048]             */
    double r = nearbyint(scaled);                     /* default mode = RNE       */
    uint32_t q = (uint32_t)r;                         /* 0 .. 2048                */
    if (e == -14 && q < 1024u) return sign | (uint16_t)q;      /* subnormal      */
    if (q == 2048u) { q = 1024u; e += 1; }
    if (e > 15) return sign | 0x7C00u;
    return sign | (uint16_t)(((uint32_t)(e + 15) << 10) | (q - 1024u));
}

static uint16_t f2h(float x) { return d2h((double)x); }

/* exported so tests can pin the conversions against numpy's float16 */
void orc_f16_to_f32(const uint16_t *h, long n, float *out)
{
    for (long i = 0; i < n; ++i) out[i] = h2f(h[i]);
}
void orc_f64_to_f16(const double *x, long n, uint16_t *out)
{
    for (long i = 0; i < n; ++i) out[i] = d2h(x[i]);
}

static int clamp_code(float r)
{
    if (r < -8.0f) return -8;
    if (r > 7.0f) return 7;
    return (int)r;
}

/* ----------------------------------------------------- weight quantizer */

/* W4 weights (unified low-bit execution form, Method overview): symmetric
 * int4 per (output row, group of `g` consecutive input channels) with an fp16
 * scale.  a = max|w|; s = fp16(a/7); a zero (or underflowed) scale becomes 1;
 * code = clamp(rne(w / s), -8, 7).  The last group may be shorter than g. */
void orc_quantize_weights(const float *w, int N, int K, int g,
                          int8_t *codes, uint16_t *scales)
{
    int G = (K + g - 1) / g;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int gi = 0; gi < G; ++gi) {
            int k0 = gi * g, k1 = k0 + g < K ? k0 + g : K;
            float a = 0.0f;
            for (int k = k0; k < k1; ++k) {
                float v = fabsf(w[(size_t)n * K + k]);
                if (v > a) a = v;
            }
            uint16_t sh = f2h(a / 7.0f);
            float s = h2f(sh);
            if (a == 0.0f || s == 0.0f) { sh = 0x3C00u; s = 1.0f; }
            scales[(size_t)n * G + gi] = sh;
            for (int k = k0; k < k1; ++k) {
                float r = rintf(w[(size_t)n * K + k] / s);
                codes[(size_t)n * K + k] = (int8_t)clamp_code(r);
            }
        }
    }
}

/* ------------------------------------------------------------- RMSNorm */

/* LLaMA-style RMSNorm in front of the quantized projections: mean square in
 * fp64, reciprocal root rounded once to fp32, then two fp32 multiplies. */
void orc_rmsnorm(const uint16_t *x, int M, int d, const float *gamma,
                 float eps, uint16_t *h)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < M; ++t) {
        const uint16_t *xr = x + (size_t)t * d;
        double ss = 0.0;
        for (int c = 0; c < d; ++c) {
            double v = (double)h2f(xr[c]);
            ss += v * v;
        }
        float rn = (float)(1.0 / sqrt(ss / (double)d + (double)eps));
        for (int c = 0; c < d; ++c) {
            float v = h2f(xr[c]) * rn;
            v = v * gamma[c];
            h[(size_t)t * d + c] = f2h(v);
        }
    }
}

/* ------------------------------------------------- activation quantizer */

/* The activation quantizer Q of the W4A4 operators, which is also the Q of
 * the low-bit risk metric (Eq. 6): per token, symmetric int4.
 *   a = max|x|, s = a/7, code = clamp(rne(x * (7/a)), -8, 7); a == 0 gives
 *   s = 1 and all-zero codes.
 * Side outputs for Eq. 6: sumsq = sum x^2 (= m_mag^2) and
 * ressq = sum (code*s - x)^2 (= m_res^2), fp64 sums rounded to fp32. */
void orc_quantize_act(const uint16_t *x, int M, int d, int8_t *q,
                      float *scale, float *sumsq, float *ressq)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < M; ++t) {
        const uint16_t *xr = x + (size_t)t * d;
        float a = 0.0f;
        double ss = 0.0;
        for (int c = 0; c < d; ++c) {
            float v = h2f(xr[c]);
            if (fabsf(v) > a) a = fabsf(v);
            ss += (double)v * (double)v;
        }
        float s = 1.0f, inv = 0.0f;
        if (a != 0.0f) { s = a / 7.0f; inv = 7.0f / a; }
        double rs = 0.0;
        for (int c = 0; c < d; ++c) {
            float v = h2f(xr[c]);
            int code = clamp_code(rintf(v * inv));
            if (q) q[(size_t)t * d + c] = (int8_t)code;
            float deq = (float)code * s;
            float r = deq - v;
            rs += (double)r * (double)r;
        }
        if (scale) scale[t] = s;
        if (sumsq) sumsq[t] = (float)ss;
        if (ressq) ressq[t] = (float)rs;
    }
}

/* ----------------------------------------------------------- W4A4 GEMM */

/* W4A4 linear operator: y[t][n] = s_a[t] * sum_g s_w[n][g] * acc_g[t][n],
 * acc_g = exact integer dot product of int4 codes over group g.  The group
 * sums are combined in fp32 with one fused multiply-add per group in
 * ascending group order, then one multiply by the token scale, one optional
 * add of the residual, one rounding to fp16.  acc_opt receives the exact
 * full-K integer dot product (no scales). */
void orc_w4a4_gemm(const int8_t *qa, const float *sa, int M, int K,
                   const int8_t *qw, const uint16_t *sw, int N, int g,
                   const uint16_t *residual, uint16_t *y, int32_t *acc_opt)
{
    int G = (K + g - 1) / g;
#pragma omp parallel for schedule(dynamic, 4)
    for (int t = 0; t < M; ++t) {
        const int8_t *ar = qa + (size_t)t * K;
        for (int n = 0; n < N; ++n) {
            const int8_t *wr = qw + (size_t)n * K;
            float y32 = 0.0f;
            int32_t total = 0;
            for (int gi = 0; gi < G; ++gi) {
                int k0 = gi * g, k1 = k0 + g < K ? k0 + g : K;
                int32_t acc = 0;
                for (int k = k0; k < k1; ++k) acc += (int32_t)ar[k] * (int32_t)wr[k];
                total += acc;
                y32 = fmaf((float)acc, h2f(sw[(size_t)n * G + gi]), y32);
            }
            float v = y32 * sa[t];
            if (residual) v = v + h2f(residual[(size_t)t * N + n]);
            if (y) y[(size_t)t * N + n] = f2h(v);
            if (acc_opt) acc_opt[(size_t)t * N + n] = total;
        }
    }
}

/* ---------------------------------------------------------------- RoPE */

/* Rotary position embedding with the rotate-half pairing (i, i + dh/2).  The
 * angle comes from caller tables indexed by the token's ORIGINAL position id,
 * so positions stay aligned with the tokens after pruning (compaction
 * paragraph after Eq. 9).  x is [M][H][dh] with row stride ldx. */
void orc_rope(const uint16_t *x, int M, int H, int dh, long ldx,
              const int32_t *pos, const float *cosT, const float *sinT,
              uint16_t *out, long ldo)
{
    int hd = dh / 2;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < M; ++t) {
        const float *c = cosT + (size_t)pos[t] * hd;
        const float *s = sinT + (size_t)pos[t] * hd;
        for (int h = 0; h < H; ++h) {
            const uint16_t *xr = x + (size_t)t * ldx + (size_t)h * dh;
            uint16_t *orow = out + (size_t)t * ldo + (size_t)h * dh;
            for (int i = 0; i < hd; ++i) {
                float x1 = h2f(xr[i]), x2 = h2f(xr[i + hd]);
                float a = x1 * c[i];
                float b = x2 * s[i];
                float e = x2 * c[i];
                float f = x1 * s[i];
                orow[i] = f2h(a - b);
                orow[i + hd] = f2h(e + f);
            }
        }
    }
}

/* ------------------------------------------------------- 4-bit KV cache */

/* 4-bit KV quantizer (quantized KV cache of the unified execution form):
 * symmetric int4 per (token, head, group of g channels), fp16 scale.
 *   a = max|x|; s = fp16(a/7) (1 if zero); code = clamp(rne(x * (1/s)));
 *   xhat = fp16(code * s) is what attention consumes.
 * x is [M][H*dh] with row stride ldx; outputs are dense. */
void orc_kv_quant(const uint16_t *x, int M, int Hdh, long ldx, int g,
                  int8_t *codes, uint16_t *scales, uint16_t *xhat)
{
    int G = Hdh / g;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < M; ++t) {
        for (int gi = 0; gi < G; ++gi) {
            const uint16_t *xr = x + (size_t)t * ldx + (size_t)gi * g;
            float a = 0.0f;
            for (int c = 0; c < g; ++c) {
                float v = fabsf(h2f(xr[c]));
                if (v > a) a = v;
            }
            uint16_t sh = f2h(a / 7.0f);
            float s = h2f(sh);
            if (a == 0.0f || s == 0.0f) { sh = 0x3C00u; s = 1.0f; }
            float r = 1.0f / s;
            if (scales) scales[(size_t)t * G + gi] = sh;
            for (int c = 0; c < g; ++c) {
                int code = clamp_code(rintf(h2f(xr[c]) * r));
                size_t o = (size_t)t * Hdh + (size_t)gi * g + c;
                if (codes) codes[o] = (int8_t)code;
                if (xhat) xhat[o] = f2h((float)code * s);
            }
        }
    }
}

/* ------------------------------------------- attention + column masses */

/* Causal softmax attention over the dequantized 4-bit K/V, straight from the
 * definition, in fp64:  S_ij = q_i . khat_j / sqrt(dh) for j <= i,
 * P = softmax_j(S), o_i = sum_j P_ij vhat_j (rounded to fp16).
 * Eq. 6 attention cues for each visual key i (A indexed [query][key]):
 *   m_inter[i] = (1/H) sum_h sum_{j in text queries}   P^h[j][i]
 *   m_intra[i] = (1/H) sum_h sum_{k in visual queries} P^h[k][i]
 * Visual tokens occupy sequence slots [vis_begin, vis_begin + Nv).
 * q, khat, vhat, o are [B][N][H][dh] dense.  cm_* are [B][Nv] fp32.
 * P_opt (tests only) receives [B][H][N][N] fp64 probabilities. */
void orc_attention(const uint16_t *q, const uint16_t *khat,
                   const uint16_t *vhat, int B, int N, int H, int Hkv, int dh,
                   int vis_begin, int Nv, uint16_t *o, float *cm_inter,
                   float *cm_intra, double *P_opt)
{
    /* grouped-query attention: query head h reads K/V head h / (H / Hkv); Hkv == H is
     * ordinary multi-head attention.  q, o have H heads per row, khat, vhat have Hkv. */
    size_t d = (size_t)H * dh, dkv = (size_t)Hkv * dh;
    int rep = H / Hkv;
    double inv_sqrt = 1.0 / sqrt((double)dh);
    /* per (b, h) column sums, reduced over heads afterwards in head order */
    double *ci = (double *)calloc((size_t)B * H * (Nv > 0 ? Nv : 1), sizeof(double));
    double *cv = (double *)calloc((size_t)B * H * (Nv > 0 ? Nv : 1), sizeof(double));
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            double *p = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
            double *acc = (double *)malloc(sizeof(double) * (size_t)dh);
            double *cih = ci + ((size_t)b * H + h) * Nv;
            double *cvh = cv + ((size_t)b * H + h) * Nv;
            for (int i = 0; i < N; ++i) {
                const uint16_t *qi = q + ((size_t)b * N + i) * d + (size_t)h * dh;
                double mx = -INFINITY;
                for (int j = 0; j <= i; ++j) {
                    const uint16_t *kj = khat + ((size_t)b * N + j) * dkv + (size_t)(h / rep) * dh;
                    double s = 0.0;
                    for (int c = 0; c < dh; ++c) s += (double)h2f(qi[c]) * (double)h2f(kj[c]);
                    s *= inv_sqrt;
                    p[j] = s;
                    if (s > mx) mx = s;
                }
                double den = 0.0;
                for (int j = 0; j <= i; ++j) { p[j] = exp(p[j] - mx); den += p[j]; }
                for (int c = 0; c < dh; ++c) acc[c] = 0.0;
                int q_is_vis = (i >= vis_begin && i < vis_begin + Nv);
                for (int j = 0; j <= i; ++j) {
                    double pj = p[j] / den;
                    const uint16_t *vj = vhat + ((size_t)b * N + j) * dkv + (size_t)(h / rep) * dh;
                    for (int c = 0; c < dh; ++c) acc[c] += pj * (double)h2f(vj[c]);
                    if (j >= vis_begin && j < vis_begin + Nv) {
                        if (q_is_vis) cvh[j - vis_begin] += pj;
                        else cih[j - vis_begin] += pj;
                    }
                    if (P_opt) P_opt[(((size_t)b * H + h) * N + i) * N + j] = pj;
                }
                if (P_opt)
                    for (int j = i + 1; j < N; ++j)
                        P_opt[(((size_t)b * H + h) * N + i) * N + j] = 0.0;
                if (o)
                    for (int c = 0; c < dh; ++c)
                        o[((size_t)b * N + i) * d + (size_t)h * dh + c] = d2h(acc[c]);
            }
            free(p);
            free(acc);
        }
    }
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < Nv; ++i) {
            double si = 0.0, sv = 0.0;
            for (int h = 0; h < H; ++h) {
                si += ci[((size_t)b * H + h) * Nv + i];
                sv += cv[((size_t)b * H + h) * Nv + i];
            }
            if (cm_inter) cm_inter[(size_t)b * Nv + i] = (float)(si / (double)H);
            if (cm_intra) cm_intra[(size_t)b * Nv + i] = (float)(sv / (double)H);
        }
    free(ci);
    free(cv);
}

/* ------------------------------------------------- scoring (Eq. 6 - 8) */

static int cmp_float(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

/* Robust per-layer normalisation G (Eq. 7) as read here: clip to the
 * [p_lo, p_hi] percentiles and rescale to [0, 1].  Percentiles are
 * nearest-rank order statistics of the Nv values of one sequence:
 * rank(p) = (p*(Nv-1) + 50) / 100 in integer arithmetic on the ascending
 * sort.  A flat metric (hi == lo) maps to 0.5 for every token. */
static void robust_norm(const float *m, int n, int p_lo, int p_hi, float *out)
{
    float *s = (float *)malloc(sizeof(float) * (size_t)n);
    memcpy(s, m, sizeof(float) * (size_t)n);
    qsort(s, (size_t)n, sizeof(float), cmp_float);
    float lo = s[(p_lo * (n - 1) + 50) / 100];
    float hi = s[(p_hi * (n - 1) + 50) / 100];
    free(s);
    for (int i = 0; i < n; ++i) {
        if (hi == lo) { out[i] = 0.5f; continue; }
        float num = m[i] - lo;
        float den = hi - lo;
        float v = num / den;
        if (v < 0.0f) v = 0.0f;
        if (v > 1.0f) v = 1.0f;
        out[i] = v;
    }
}

/* Composite score (Eq. 8) from the four Eq. 6 metrics:
 *   m_mag = sqrt(sumsq), m_res = sqrt(ressq) (fp32 square roots of the
 *   quantizer's side outputs), m_inter / m_intra = attention column masses.
 * Each metric is normalised per sequence with G (Eq. 7), then
 *   score = ((w_m*g_mag + w_c*g_inter) + w_s*g_intra) + w_r*g_res
 * in fp32, each product and sum rounded separately.  All arrays [B][Nv].
 * normed_opt receives [4][B][Nv] in the order mag, inter, intra, res. */
void orc_score(const float *sumsq, const float *ressq, const float *cm_inter,
               const float *cm_intra, int B, int Nv, float w_m, float w_c,
               float w_s, float w_r, int p_lo, int p_hi, float *score,
               float *normed_opt)
{
    if (Nv <= 0) return;
    float *tmp = (float *)malloc(sizeof(float) * (size_t)Nv * 5);
    float *raw = tmp, *g[4] = {tmp + Nv, tmp + 2 * Nv, tmp + 3 * Nv, tmp + 4 * Nv};
    for (int b = 0; b < B; ++b) {
        size_t o = (size_t)b * Nv;
        for (int i = 0; i < Nv; ++i) raw[i] = sqrtf(sumsq[o + i]);
        robust_norm(raw, Nv, p_lo, p_hi, g[0]);
        robust_norm(cm_inter + o, Nv, p_lo, p_hi, g[1]);
        robust_norm(cm_intra + o, Nv, p_lo, p_hi, g[2]);
        for (int i = 0; i < Nv; ++i) raw[i] = sqrtf(ressq[o + i]);
        robust_norm(raw, Nv, p_lo, p_hi, g[3]);
        for (int i = 0; i < Nv; ++i) {
            float a = w_m * g[0][i];
            float c = w_c * g[1][i];
            float s = w_s * g[2][i];
            float r = w_r * g[3][i];
            float acc = a + c;
            acc = acc + s;
            acc = acc + r;
            score[o + i] = acc;
        }
        if (normed_opt)
            for (int k = 0; k < 4; ++k)
                memcpy(normed_opt + ((size_t)k * B + b) * Nv, g[k], sizeof(float) * (size_t)Nv);
    }
    free(tmp);
}

/* ------------------------------------------------------- top-k (Eq. 9) */

typedef struct { float s; int32_t i; } scored_t;

static int cmp_scored(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    int xn = x->s != x->s, yn = y->s != y->s;      /* NaN ranks lowest */
    if (xn != yn) return xn - yn;
    if (!xn) {
        if (x->s > y->s) return -1;
        if (x->s < y->s) return 1;
    }
    return (x->i > y->i) - (x->i < y->i);
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Deterministic TopK (Eq. 9): full sort by (score descending, index
 * ascending), take the first min(K, Nv), emit them in ascending index order.
 * keep_idx is [B][min(K, Nv)]. */
void orc_topk(const float *score, int B, int Nv, int K, int32_t *keep_idx)
{
    int k = K < Nv ? K : Nv;
    if (k <= 0) return;
    scored_t *v = (scored_t *)malloc(sizeof(scored_t) * (size_t)Nv);
    for (int b = 0; b < B; ++b) {
        for (int i = 0; i < Nv; ++i) { v[i].s = score[(size_t)b * Nv + i]; v[i].i = i; }
        qsort(v, (size_t)Nv, sizeof(scored_t), cmp_scored);
        int32_t *out = keep_idx + (size_t)b * k;
        for (int i = 0; i < k; ++i) out[i] = v[i].i;
        qsort(out, (size_t)k, sizeof(int32_t), cmp_i32);
    }
    free(v);
}

/* ------------------------------------------------------ SwiGLU product */

/* z = fp16(silu(gate) * up), silu(x) = x / (1 + exp(-x)), evaluated in fp64
 * and rounded once.  gu is [M][2F]: gate in columns [0,F), up in [F,2F). */
void orc_silu_mul(const uint16_t *gu, int M, int F, uint16_t *z)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < M; ++t)
        for (int c = 0; c < F; ++c) {
            double gt = (double)h2f(gu[(size_t)t * 2 * F + c]);
            double up = (double)h2f(gu[(size_t)t * 2 * F + F + c]);
            z[(size_t)t * F + c] = d2h(gt / (1.0 + exp(-gt)) * up);
        }
}
