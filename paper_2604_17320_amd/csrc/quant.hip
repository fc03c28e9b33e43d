// Quantizers of the W4A4 execution form: weight group quantizer + repack,
// per-token int4 activation quantizer (the Q of Eq. 6) and its fused variants
// (RMSNorm in front of QKV / gate-up, SwiGLU product in front of down).
// All are row kernels: one wave per row (four rows per workgroup) up to 4096
// columns, one workgroup per row beyond; the row is cached in registers as
// 16-byte chunks, absmax / sums of squares are wave or block reductions, one
// packed dword (8 codes) is stored per chunk.  HBM-bound by design.
#include "common.h"
#include "internal.h"
#include "rowquant.h"

// ------------------------------------------------------------ W4 weights

// one wave per (row n, group g): 2 elements per lane
__global__ __launch_bounds__(256) void quantize_weights_kernel(
    const float *__restrict__ w, int N, int K, int G, int8_t *__restrict__ codes,
    f16 *__restrict__ scales)
{
    long wave = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (wave >= (long)N * G) return;
    int n = (int)(wave / G), g = (int)(wave % G);
    int k = g * QUOTA_GROUP_W + 2 * lane;
    const float *wr = w + (size_t)n * K;
    float v0 = k < K ? wr[k] : 0.0f;
    float v1 = k + 1 < K ? wr[k + 1] : 0.0f;
    float a = wave_max(fmaxf(fabsf(v0), fabsf(v1)));
    f16 sh = to_f16(a / 7.0f);
    float s = (float)sh;
    if (a == 0.0f || s == 0.0f) { sh = (f16)1.0f; s = 1.0f; }
    if (lane == 0) scales[(size_t)n * G + g] = sh;
    if (k < K) codes[(size_t)n * K + k] = (int8_t)code_from(rintf(v0 / s));
    if (k + 1 < K) codes[(size_t)n * K + k + 1] = (int8_t)code_from(rintf(v1 / s));
}

// codes int8 [N][K] -> packed [G][N][16 dwords]; scales [N][G] -> [G][N]
__global__ __launch_bounds__(256) void pack_weights_kernel(
    const int8_t *__restrict__ codes, const f16 *__restrict__ scales, int N, int K, int G,
    uint32_t *__restrict__ packed, f16 *__restrict__ scales_t)
{
    long t = (long)blockIdx.x * 256 + threadIdx.x;
    long total = (long)G * N * 16;
    if (t >= total) return;
    int i = (int)(t & 15);
    long gn = t >> 4;
    int n = (int)(gn % N), g = (int)(gn / N);
    int k0 = g * QUOTA_GROUP_W + 8 * i;
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        int k = k0 + e;
        int c = k < K ? (int)codes[(size_t)n * K + k] : 0;
        word |= (uint32_t)(c & 0xF) << (4 * e);
    }
    packed[t] = word;
    if (i == 0) scales_t[(size_t)g * N + n] = scales[(size_t)n * G + g];
}

// ------------------------------------------------- activation quantizers

// A row is owned by GROUP threads, each caching NCH chunks (2 or 8).  Every load of a thread is
// issued before the first use (unconditional loads at clamped indices instead of guarded ones, so
// that nothing separates them): one memory round trip per kernel.  GROUP = 64 (rows of up to 4096
// columns): one WAVE per row, four rows per workgroup -- a lane issues all its 16-byte loads back
// to back, the reductions are wave shuffles and there is no workgroup barrier.  GROUP = 256 (up to
// 16384 columns): the whole workgroup owns the row and reduces through LDS.
// Below this many rows the launch cannot fill the chip with one wave per row, and a row is
// finished sooner by a whole workgroup.
#define ROW_WAVE_MIN_ROWS 2048

template <int GROUP>
__device__ __forceinline__ void group_reduce(float &mx, double &s0, double &s1, double *sm)
{
    if (GROUP == 64) { mx = wave_max(mx); s0 = wave_sum(s0); s1 = wave_sum(s1); }
    else block_max_sum2<4>(mx, s0, s1, sm);
}
#define ROW_PROLOGUE()                                                                         \
    __shared__ double sm[12];                                                                  \
    const int lane = threadIdx.x % GROUP;                                                      \
    const int row = blockIdx.x * (ROW_THREADS / GROUP) + threadIdx.x / GROUP;                  \
    if (row >= M) return;     /* GROUP = 64: the whole wave leaves; GROUP = 256: never taken */ \
    (void)sm

template <bool WANT_METRICS, int GROUP, int NCH>
__global__ __launch_bounds__(ROW_THREADS) void quantize_act_kernel(
    const f16 *__restrict__ x, int M, int d, long ldx, int rows_per_seq, long seq_stride,
    uint32_t *__restrict__ q, float *__restrict__ scale, float *__restrict__ sumsq,
    float *__restrict__ ressq)
{
    ROW_PROLOGUE();
    const int nchunk = d >> 3;
    const uint4 *xr = reinterpret_cast<const uint4 *>(
        x + (size_t)(row / rows_per_seq) * seq_stride + (size_t)(row % rows_per_seq) * ldx);
    Pack16 v[NCH];
    float a = 0.0f;
    double ss = 0.0;
#pragma unroll
    for (int r = 0; r < NCH; ++r) v[r].u = xr[min(lane + GROUP * r, nchunk - 1)];
#pragma unroll
    for (int r = 0; r < NCH; ++r) {
        int c = lane + GROUP * r;
        if (c < nchunk) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f = (float)v[r].h[e];
                a = fmaxf(a, fabsf(f));
                if (WANT_METRICS) ss = __builtin_fma((double)f, (double)f, ss);     // product exact in fp64
            }
        }
    }
    double zero = 0.0;
    group_reduce<GROUP>(a, ss, zero, sm);
    float s;
    double rs = quantize_cached_row<WANT_METRICS, GROUP, NCH>(v, nchunk, lane, a,
                                                              q ? q + (size_t)row * nchunk : nullptr, s);
    if (WANT_METRICS) { float dummy = 0.0f; group_reduce<GROUP>(dummy, rs, zero, sm); }
    if (lane == 0) {
        if (scale) scale[row] = s;
        if (WANT_METRICS) {
            if (sumsq) sumsq[row] = (float)ss;
            if (ressq) ressq[row] = (float)rs;
        }
    }
}

template <bool WANT_METRICS, int GROUP, int NCH>
__global__ __launch_bounds__(ROW_THREADS) void rmsnorm_quantize_act_kernel(
    const f16 *__restrict__ x, int M, int d, long ldx, const float *__restrict__ gamma, float eps,
    uint32_t *__restrict__ q, float *__restrict__ scale, float *__restrict__ sumsq,
    float *__restrict__ ressq, f16 *__restrict__ h_out)
{
    ROW_PROLOGUE();
    const int nchunk = d >> 3;
    const uint4 *xr = reinterpret_cast<const uint4 *>(x + (size_t)row * ldx);
    Pack16 v[NCH];
    float a_raw = 0.0f;
    double ss = 0.0;
    // wave-per-row launches are long (thousands of rows): the gains are fetched where they are used
    // (they stay in cache) so that more waves fit on a SIMD; workgroup-per-row launches are short and
    // latency counts, so there every load is issued up front
    constexpr bool GAINS_EARLY = GROUP != 64;
    float4 ga[GAINS_EARLY ? NCH : 1][2];
#pragma unroll
    for (int r = 0; r < NCH; ++r) {
        const int c = min(lane + GROUP * r, nchunk - 1);
        v[r].u = xr[c];
        if (GAINS_EARLY) {
            const float4 *gp = reinterpret_cast<const float4 *>(gamma + 8 * c);
            ga[r][0] = gp[0];
            ga[r][1] = gp[1];
        }
    }
#pragma unroll
    for (int r = 0; r < NCH; ++r) {
        int c = lane + GROUP * r;
        if (c < nchunk) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f = (float)v[r].h[e];
                a_raw = fmaxf(a_raw, fabsf(f));
                ss = __builtin_fma((double)f, (double)f, ss);     // product exact in fp64
            }
        }
    }
    double zero = 0.0;
    group_reduce<GROUP>(a_raw, ss, zero, sm);
    if (!GAINS_EARLY) {
        // the row stays packed (32 registers for 4096 columns): without this the compiler keeps the 64
        // converted floats of the first pass alive for the second one
#pragma unroll
        for (int r = 0; r < NCH; ++r)
            asm volatile("" : "+v"(v[r].u.x), "+v"(v[r].u.y), "+v"(v[r].u.z), "+v"(v[r].u.w));
    }
    float rn = (float)(1.0 / sqrt(ss / (double)d + (double)eps));
    float s_raw = 1.0f, inv_raw = 0.0f;
    if (a_raw != 0.0f) { s_raw = a_raw / 7.0f; inv_raw = 7.0f / a_raw; }
    float a = 0.0f;
    double rs = 0.0;
#pragma unroll
    for (int r = 0; r < NCH; ++r) {
        int c = lane + GROUP * r;
        if (c < nchunk) {
            const float4 *gp = reinterpret_cast<const float4 *>(gamma + 8 * c);
            const float4 g0 = GAINS_EARLY ? ga[GAINS_EARLY ? r : 0][0] : gp[0];
            const float4 g1 = GAINS_EARLY ? ga[GAINS_EARLY ? r : 0][1] : gp[1];
            float gm[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f = (float)v[r].h[e];
                if (WANT_METRICS) {
                    float deq = code_float(code_bits(f * inv_raw)) * s_raw;
                    float rr = deq - f;
                    rs = __builtin_fma((double)rr, (double)rr, rs);
                }
                float hn = f * rn;
                hn = hn * gm[e];
                f16 hh = to_f16(hn);
                v[r].h[e] = hh;
                a = fmaxf(a, fabsf((float)hh));
            }
            if (h_out) reinterpret_cast<uint4 *>(h_out + (size_t)row * d)[c] = v[r].u;
        }
        // keep the compiler from hoisting every chunk's gain loads to the top (that costs 64 registers)
        if (!GAINS_EARLY) __builtin_amdgcn_sched_barrier(0);
    }
    group_reduce<GROUP>(a, rs, zero, sm);
    float s;
    quantize_cached_row<false, GROUP, NCH>(v, nchunk, lane, a, q + (size_t)row * nchunk, s);
    if (lane == 0) {
        scale[row] = s;
        if (WANT_METRICS) {
            if (sumsq) sumsq[row] = (float)ss;
            if (ressq) ressq[row] = (float)rs;
        }
    }
}

// EARLY: every load before the first use (short launches, latency counts); otherwise chunk by
// chunk (long launches: fewer live registers, more waves per SIMD to hide the latency instead).
template <int GROUP, int NCH, bool EARLY>
__global__ __launch_bounds__(ROW_THREADS) void silu_mul_quantize_act_kernel(
    const f16 *__restrict__ gu, int M, int F, uint32_t *__restrict__ q, float *__restrict__ scale,
    f16 *__restrict__ z_out, const f16 *__restrict__ z_inject)
{
    ROW_PROLOGUE();
    const int nchunk = F >> 3;
    const uint4 *gr = reinterpret_cast<const uint4 *>(gu + (size_t)row * 2 * F);
    const uint4 *ur = reinterpret_cast<const uint4 *>(gu + (size_t)row * 2 * F + F);
    Pack16 v[NCH], gg[NCH], uu[NCH];
    float a = 0.0f;
    if (z_inject) {
#pragma unroll
        for (int r = 0; r < NCH; ++r)
            v[r].u = reinterpret_cast<const uint4 *>(z_inject + (size_t)row * F)[min(lane + GROUP * r, nchunk - 1)];
    } else if (EARLY) {
#pragma unroll
        for (int r = 0; r < NCH; ++r) {
            const int c = min(lane + GROUP * r, nchunk - 1);
            gg[r].u = gr[c];
            uu[r].u = ur[c];
        }
    }
#pragma unroll
    for (int r = 0; r < NCH; ++r) {
        int c = lane + GROUP * r;
        if (c < nchunk) {
            if (!z_inject) {
                if (!EARLY) { gg[r].u = gr[c]; uu[r].u = ur[c]; }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float gt = (float)gg[r].h[e], up = (float)uu[r].h[e];
                    // silu(g) = g / (1 + e^-g) with the hardware exp2 and reciprocal (a few fp32 ulp,
                    // far inside the fp16 rounding that follows)
                    float sg = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt));
                    v[r].h[e] = to_f16(sg * up);
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf((float)v[r].h[e]));
            if (z_out) reinterpret_cast<uint4 *>(z_out + (size_t)row * F)[c] = v[r].u;
        }
    }
    double z0 = 0.0, z1 = 0.0;
    group_reduce<GROUP>(a, z0, z1, sm);
    float s;
    quantize_cached_row<false, GROUP, NCH>(v, nchunk, lane, a, q + (size_t)row * nchunk, s);
    if (lane == 0) scale[row] = s;
}

// ------------------------------------------------------------ host side

extern "C" size_t quota_weights_packed_bytes(int N, int K)
{
    if (N <= 0 || K <= 0) return 0;
    size_t G = ((size_t)K + QUOTA_GROUP_W - 1) / QUOTA_GROUP_W;
    return G * (size_t)N * 64;
}

extern "C" size_t quota_weights_scale_bytes(int N, int K)
{
    if (N <= 0 || K <= 0) return 0;
    size_t G = ((size_t)K + QUOTA_GROUP_W - 1) / QUOTA_GROUP_W;
    return G * (size_t)N * 2;
}

extern "C" int quota_quantize_weights(const float *w, int N, int K, int8_t *codes,
                                      void *scales_f16, void *stream)
{
    if (!w || !codes || !scales_f16) return QUOTA_ERR_NULL;
    if (N <= 0 || K <= 0) return QUOTA_ERR_INVALID_ARG;
    int G = (K + QUOTA_GROUP_W - 1) / QUOTA_GROUP_W;
    long waves = (long)N * G;
    ProfScope prof(QUOTA_K_QUANTIZE_WEIGHTS, 0, 5.0 * N * K + 2.0 * N * G, (hipStream_t)stream);
    quantize_weights_kernel<<<dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, (hipStream_t)stream>>>(
        w, N, K, G, codes, (f16 *)scales_f16);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" int quota_pack_weights(const int8_t *codes, const void *scales_f16,
                                  const quota_weights *W, void *stream)
{
    if (!codes || !scales_f16 || !W || !W->packed || !W->scales) return QUOTA_ERR_NULL;
    if (W->N <= 0 || W->K <= 0) return QUOTA_ERR_INVALID_ARG;
    if (W->N % 64 != 0 || W->K % 32 != 0) return QUOTA_ERR_SHAPE;
    int G = (W->K + QUOTA_GROUP_W - 1) / QUOTA_GROUP_W;
    long total = (long)G * W->N * 16;
    ProfScope prof(QUOTA_K_PACK_WEIGHTS, 0, 1.5 * W->N * W->K + 4.0 * W->N * G, (hipStream_t)stream);
    pack_weights_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
        codes, (const f16 *)scales_f16, W->N, W->K, G, (uint32_t *)W->packed, (f16 *)W->scales);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

static int check_rows(const void *x, int M, int d, int ld, const void *q, const void *scale)
{
    if (!x || !q || !scale) return QUOTA_ERR_NULL;
    if (M < 0 || d <= 0) return QUOTA_ERR_INVALID_ARG;
    if (d % 8 != 0 || d > ROW_MAXCOLS || ld < d || ld % 8 != 0) return QUOTA_ERR_SHAPE;
    return QUOTA_OK;
}

extern "C" int quota_quantize_act(const void *x_f16, int M, int d, int ldx, uint8_t *q_packed,
                                  float *scale, float *sumsq_opt, float *ressq_opt, void *stream)
{
    int rc = check_rows(x_f16, M, d, ldx, q_packed, scale);
    if (rc != QUOTA_OK) return rc;
    if (M == 0) return QUOTA_OK;
    hipStream_t st = (hipStream_t)stream;
    ProfScope prof(QUOTA_K_QUANTIZE_ACT, 0, 2.5 * M * d + 4.0 * M, st);
    const bool metrics = sumsq_opt || ressq_opt, small = d <= 4096 && M >= ROW_WAVE_MIN_ROWS;
    const dim3 grid(small ? (M + 3) / 4 : M), blk(ROW_THREADS);
    const f16 *x = (const f16 *)x_f16;
    uint32_t *q = (uint32_t *)q_packed;
    const bool few = (d >> 3) <= 2 * (small ? 64 : 256);      // two chunks per thread are enough
    const bool many = d > 16384;                              // sixteen chunks per thread
#define QUOTA_LAUNCH_Q(MET, GRP, NCH) \
    quantize_act_kernel<MET, GRP, NCH><<<grid, blk, 0, st>>>(x, M, d, ldx, M, 0, q, scale, sumsq_opt, ressq_opt)
    if (metrics) {
        if (small) { if (few) QUOTA_LAUNCH_Q(true, 64, 2); else QUOTA_LAUNCH_Q(true, 64, 8); }
        else if (many) QUOTA_LAUNCH_Q(true, 256, 16);
        else { if (few) QUOTA_LAUNCH_Q(true, 256, 2); else QUOTA_LAUNCH_Q(true, 256, 8); }
    } else {
        if (small) { if (few) QUOTA_LAUNCH_Q(false, 64, 2); else QUOTA_LAUNCH_Q(false, 64, 8); }
        else if (many) QUOTA_LAUNCH_Q(false, 256, 16);
        else { if (few) QUOTA_LAUNCH_Q(false, 256, 2); else QUOTA_LAUNCH_Q(false, 256, 8); }
    }
#undef QUOTA_LAUNCH_Q
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" int quota_rmsnorm_quantize_act(const void *x_f16, int M, int d, int ldx,
                                          const float *gamma, float eps, uint8_t *q_packed,
                                          float *scale, float *sumsq_opt, float *ressq_opt,
                                          void *h_opt, void *stream)
{
    int rc = check_rows(x_f16, M, d, ldx, q_packed, scale);
    if (rc != QUOTA_OK) return rc;
    if (!gamma) return QUOTA_ERR_NULL;
    if (!(eps >= 0.0f)) return QUOTA_ERR_INVALID_ARG;
    if (M == 0) return QUOTA_OK;
    hipStream_t st = (hipStream_t)stream;
    ProfScope prof(QUOTA_K_RMSNORM_QUANTIZE_ACT, 0, 2.5 * M * d + 4.0 * M + 4.0 * d, st);
    const bool metrics = sumsq_opt || ressq_opt, small = d <= 4096 && M >= ROW_WAVE_MIN_ROWS;
    const dim3 grid(small ? (M + 3) / 4 : M), blk(ROW_THREADS);
    const f16 *x = (const f16 *)x_f16;
    uint32_t *q = (uint32_t *)q_packed;
    f16 *h = (f16 *)h_opt;
    const bool few = (d >> 3) <= 2 * (small ? 64 : 256);      // two chunks per thread are enough
    const bool many = d > 16384;                              // sixteen chunks per thread
#define QUOTA_LAUNCH_R(MET, GRP, NCH)                                                                  \
    rmsnorm_quantize_act_kernel<MET, GRP, NCH><<<grid, blk, 0, st>>>(x, M, d, ldx, gamma, eps, q, scale, \
                                                                     sumsq_opt, ressq_opt, h)
    if (metrics) {
        if (small) { if (few) QUOTA_LAUNCH_R(true, 64, 2); else QUOTA_LAUNCH_R(true, 64, 8); }
        else if (many) QUOTA_LAUNCH_R(true, 256, 16);
        else { if (few) QUOTA_LAUNCH_R(true, 256, 2); else QUOTA_LAUNCH_R(true, 256, 8); }
    } else {
        if (small) { if (few) QUOTA_LAUNCH_R(false, 64, 2); else QUOTA_LAUNCH_R(false, 64, 8); }
        else if (many) QUOTA_LAUNCH_R(false, 256, 16);
        else { if (few) QUOTA_LAUNCH_R(false, 256, 2); else QUOTA_LAUNCH_R(false, 256, 8); }
    }
#undef QUOTA_LAUNCH_R
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" int quota_silu_mul_quantize_act(const void *gu_f16, int M, int F, uint8_t *q_packed,
                                           float *scale, void *z_opt, const void *z_inject_opt,
                                           void *stream)
{
    int rc = check_rows(gu_f16, M, F, F, q_packed, scale);
    if (rc != QUOTA_OK) return rc;
    if (M == 0) return QUOTA_OK;
    ProfScope prof(QUOTA_K_SILU_MUL_QUANTIZE_ACT, 0, 4.5 * M * F + 4.0 * M, (hipStream_t)stream);
    const bool small = F <= 4096 && M >= ROW_WAVE_MIN_ROWS;
    const dim3 grid(small ? (M + 3) / 4 : M), blk(ROW_THREADS);
    const bool few = (F >> 3) <= 2 * (small ? 64 : 256);
    const bool many = F > 16384;          // sixteen chunks per thread, loaded chunk by chunk
#define QUOTA_LAUNCH_S(GRP, NCH, EARLY)                                                               \
    silu_mul_quantize_act_kernel<GRP, NCH, EARLY><<<grid, blk, 0, (hipStream_t)stream>>>(             \
        (const f16 *)gu_f16, M, F, (uint32_t *)q_packed, scale, (f16 *)z_opt, (const f16 *)z_inject_opt)
    if (many) QUOTA_LAUNCH_S(256, 16, false);
    else if (M >= ROW_WAVE_MIN_ROWS) {
        if (small) { if (few) QUOTA_LAUNCH_S(64, 2, false); else QUOTA_LAUNCH_S(64, 8, false); }
        else { if (few) QUOTA_LAUNCH_S(256, 2, false); else QUOTA_LAUNCH_S(256, 8, false); }
    } else {
        if (small) { if (few) QUOTA_LAUNCH_S(64, 2, true); else QUOTA_LAUNCH_S(64, 8, true); }
        else { if (few) QUOTA_LAUNCH_S(256, 2, true); else QUOTA_LAUNCH_S(256, 8, true); }
    }
#undef QUOTA_LAUNCH_S
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

// Eq. 6 vector metrics only (no codes stored): sumsq/ressq [B][Nv] of the
// visual rows v[b][i] = v + b*stride_b + i*ldv.
int quota_internal_vector_metrics(const void *v_f16, int B, int Nv, int d, int ldv, long stride_b,
                                  float *sumsq, float *ressq, hipStream_t st)
{
    if (!v_f16 || !sumsq || !ressq) return QUOTA_ERR_NULL;
    if (B <= 0 || Nv < 0 || d <= 0) return QUOTA_ERR_INVALID_ARG;
    if (d % 8 != 0 || d > ROW_MAXCOLS || ldv < d || ldv % 8 != 0 || stride_b % 8 != 0)
        return QUOTA_ERR_SHAPE;
    if (Nv == 0) return QUOTA_OK;
    ProfScope prof(QUOTA_K_QUANTIZE_ACT, 0, 2.0 * B * Nv * d + 8.0 * B * Nv, st);
    const bool small = d <= 4096 && B * Nv >= ROW_WAVE_MIN_ROWS;
    const dim3 grid(small ? (B * Nv + 3) / 4 : B * Nv), blk(ROW_THREADS);
    const bool few = (d >> 3) <= 2 * (small ? 64 : 256);
#define QUOTA_LAUNCH_V(GRP, NCH)                                                                           \
    quantize_act_kernel<true, GRP, NCH><<<grid, blk, 0, st>>>((const f16 *)v_f16, B * Nv, d, ldv, Nv, stride_b, \
                                                              nullptr, nullptr, sumsq, ressq)
    if (small) { if (few) QUOTA_LAUNCH_V(64, 2); else QUOTA_LAUNCH_V(64, 8); }
    else if (d > 16384) QUOTA_LAUNCH_V(256, 16);
    else { if (few) QUOTA_LAUNCH_V(256, 2); else QUOTA_LAUNCH_V(256, 8); }
#undef QUOTA_LAUNCH_V
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}
