// Sensitivity profiling for the offline allocator (Eq. 1): the full-precision counterpart of a
// decoder block -- fp16 storage, fp32 accumulation, no quantizer anywhere -- the per-sample
// deviation norms ||x^q - x||_2 and ||x||_2, and the call that runs a block both ways on one
// input.  This is calibration-time code, outside the deployed forward pass: the kernels are
// plain (the GEMM reads its operands straight from global memory into fp16 MFMA fragments) and
// are not tuned.
#include "common.h"
#include "internal.h"

namespace {

// ---- y = x W^T (+ residual): fp16 operands, fp32 accumulation, fp16 result ------------------
// A workgroup of 4 waves covers 128 x 128 outputs, a wave 64 x 64 as 2 x 2 tiles of
// v_mfma_f32_32x32x16_f16.  Lane l supplies 8 consecutive k of row (l % 32) to both operands
// (k slots 8 (l / 32) .. +7 of the step), and receives column l % 32 of the tile, rows
// 8 (r / 4) + 4 (l / 32) + r % 4 for r = 0..15.  Rows beyond M are read from row M - 1 and not
// stored.  Needs N % 64 == 0, K % 16 == 0.
__global__ __launch_bounds__(256) void fp_gemm_kernel(const f16 *__restrict__ x, int M, int K,
                                                       const f16 *__restrict__ W, int N,
                                                       const f16 *__restrict__ residual,
                                                       f16 *__restrict__ y)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m0 = blockIdx.y * 128 + (wave >> 1) * 64, n0 = blockIdx.x * 128 + (wave & 1) * 64;
    if (m0 >= M || n0 >= N) return;
    const int l32 = lane & 31, half = lane >> 5;
    const f16 *pa[2], *pb[2];
    for (int i = 0; i < 2; ++i) {
        const int row = min(m0 + 32 * i + l32, M - 1);
        pa[i] = x + (size_t)row * K + 8 * half;
        pb[i] = W + (size_t)(n0 + 32 * i + l32) * K + 8 * half;
    }
    f32x16 acc[2][2];
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j)
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    for (int k0 = 0; k0 < K; k0 += 16) {
        f16x8 a[2], b[2];
        for (int i = 0; i < 2; ++i) {
            a[i] = *(const f16x8 *)(pa[i] + k0);
            b[i] = *(const f16x8 *)(pb[i] + k0);
        }
        for (int i = 0; i < 2; ++i)
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j)
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
                const int col = n0 + 32 * j + l32;
                if (row < M) {
                    float v = acc[i][j][r];
                    if (residual) v += (float)residual[(size_t)row * N + col];
                    y[(size_t)row * N + col] = (f16)v;
                }
            }
}

// ---- h = x / sqrt(mean(x^2) + eps) * gamma, one workgroup per row ------------------------------
__global__ __launch_bounds__(256) void fp_rmsnorm_kernel(const f16 *__restrict__ x, int d,
                                                          const float *__restrict__ gamma, float eps,
                                                          f16 *__restrict__ h)
{
    __shared__ float part[4];
    const f16 *row = x + (size_t)blockIdx.x * d;
    float s = 0.0f;
    for (int c = threadIdx.x; c < d; c += 256) {
        const float v = (float)row[c];
        s += v * v;
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    const float inv = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += 256)
        h[(size_t)blockIdx.x * d + c] = (f16)((float)row[c] * inv * gamma[c]);
}

// ---- rotate-half RoPE of q and k at the tokens' position ids; v is copied --------------------
// qkv [M][d + 2 dkv] -> q [M][d], k [M][dkv], v [M][dkv].  One thread per (row, pair) of q | k and
// per element pair of v.
__global__ __launch_bounds__(256) void fp_rope_kernel(const f16 *__restrict__ qkv, int M, int d, int dkv,
                                                       int dh, const int32_t *__restrict__ pos,
                                                       const float *__restrict__ cosT,
                                                       const float *__restrict__ sinT, int n_pos,
                                                       f16 *__restrict__ q, f16 *__restrict__ k,
                                                       f16 *__restrict__ v)
{
    const int hd = dh / 2, per_row = (d + 2 * dkv) / 2;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)M * per_row) return;
    const int m = (int)(idx / per_row), t = (int)(idx % per_row);
    const f16 *src = qkv + (size_t)m * (d + 2 * dkv);
    if (t < (d + dkv) / 2) {                       // a rotated pair of q or k
        const int head = t / hd, i = t % hd;
        const int p = min(max(pos[m], 0), n_pos - 1);
        const float c = cosT[(size_t)p * hd + i], s = sinT[(size_t)p * hd + i];
        const float lo = (float)src[head * dh + i], hi = (float)src[head * dh + i + hd];
        const f16 rlo = (f16)(lo * c - hi * s), rhi = (f16)(hi * c + lo * s);
        const int col = head * dh + i;
        if (col < d) {
            q[(size_t)m * d + col] = rlo;
            q[(size_t)m * d + col + hd] = rhi;
        } else {
            k[(size_t)m * dkv + col - d] = rlo;
            k[(size_t)m * dkv + col - d + hd] = rhi;
        }
    } else {
        const int e = 2 * (t - (d + dkv) / 2);
        v[(size_t)m * dkv + e] = src[d + dkv + e];
        v[(size_t)m * dkv + e + 1] = src[d + dkv + e + 1];
    }
}

// ---- z = silu(gate) * up, gu [M][2F] rows gate | up ------------------------------------------
__global__ __launch_bounds__(256) void fp_silu_mul_kernel(const f16 *__restrict__ gu, long M, int F,
                                                           f16 *__restrict__ z)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * F) return;
    const long m = idx / F;
    const int f = (int)(idx % F);
    const float g = (float)gu[m * 2 * F + f], u = (float)gu[m * 2 * F + F + f];
    z[idx] = (f16)(g / (1.0f + expf(-g)) * u);
}

// ---- Eq. 1 per sample: ||x^q - x||_2 and ||x||_2 over the n values of sample blockIdx.x --------
__global__ __launch_bounds__(1024) void deviation_kernel(const f16 *__restrict__ xq,
                                                          const f16 *__restrict__ x, long n,
                                                          double *__restrict__ diff_norm,
                                                          double *__restrict__ ref_norm)
{
    __shared__ double part[2][16];
    const f16 *a = xq + (size_t)blockIdx.x * n, *b = x + (size_t)blockIdx.x * n;
    double sd = 0.0, sr = 0.0;
    for (long i = threadIdx.x; i < n; i += 1024) {
        const double r = (double)(float)b[i], e = (double)(float)a[i] - r;
        sd += e * e;
        sr += r * r;
    }
    sd = wave_sum(sd);
    sr = wave_sum(sr);
    if ((threadIdx.x & 63) == 0) {
        part[0][threadIdx.x >> 6] = sd;
        part[1][threadIdx.x >> 6] = sr;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double td = 0.0, tr = 0.0;
        for (int w = 0; w < 16; ++w) {
            td += part[0][w];
            tr += part[1][w];
        }
        diff_norm[blockIdx.x] = sqrt(td);
        ref_norm[blockIdx.x] = sqrt(tr);
    }
}

inline size_t up256(size_t n) { return (n + 255) & ~(size_t)255; }

int fp_gemm(const f16 *x, int M, int K, const void *W, int N, const f16 *residual, f16 *y, hipStream_t st)
{
    fp_gemm_kernel<<<dim3((N + 127) / 128, (M + 127) / 128), dim3(256), 0, st>>>(x, M, K, (const f16 *)W, N,
                                                                                residual, y);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

int check_fp_layer(const quota_fp_layer *L, int B, int N)
{
    if (!L) return QUOTA_ERR_NULL;
    if (!L->gamma1 || !L->gamma2 || !L->cosT || !L->sinT || !L->wqkv || !L->wo || !L->wgu || !L->wdown)
        return QUOTA_ERR_NULL;
    if (B <= 0 || N <= 0 || L->H <= 0 || L->F <= 0 || L->n_pos <= 0 || !(L->eps >= 0.0f)) return QUOTA_ERR_INVALID_ARG;
    const int Hkv = L->Hkv > 0 ? L->Hkv : L->H;
    if ((L->dh != 64 && L->dh != 128) || L->H % Hkv != 0 || L->F % 32 != 0) return QUOTA_ERR_SHAPE;
    return QUOTA_OK;
}

struct FpWs {
    f16 *h, *qkv, *q, *k, *v, *o, *x1, *gu, *z;
    void *attn;
    size_t bytes;
};

FpWs carve_fp(void *ws, const quota_fp_layer *L, int B, int N)
{
    const int Hkv = L->Hkv > 0 ? L->Hkv : L->H;
    const size_t M = (size_t)B * N, d = (size_t)L->H * L->dh, dkv = (size_t)Hkv * L->dh, F = L->F;
    char *p = (char *)ws;
    FpWs w;
    auto take = [&](size_t bytes) { void *r = p; p += up256(bytes); return r; };
    w.h = (f16 *)take(M * d * 2);
    w.qkv = (f16 *)take(M * (d + 2 * dkv) * 2);
    w.q = (f16 *)take(M * d * 2);
    w.k = (f16 *)take(M * dkv * 2);
    w.v = (f16 *)take(M * dkv * 2);
    w.o = (f16 *)take(M * d * 2);
    w.x1 = (f16 *)take(M * d * 2);
    w.gu = (f16 *)take(M * 2 * F * 2);
    w.z = (f16 *)take(M * F * 2);
    w.attn = take(quota_attention_workspace_bytes(B, N, L->H, L->dh));
    w.bytes = (size_t)(p - (char *)ws);
    return w;
}

}  // namespace

extern "C" size_t quota_fp_block_workspace_bytes(const quota_fp_layer *L, int B, int N)
{
    if (check_fp_layer(L, B, N) != QUOTA_OK) return 0;
    return carve_fp(nullptr, L, B, N).bytes;
}

extern "C" int quota_fp_block(const quota_fp_layer *L, const void *x_f16, const int32_t *pos, int B, int N,
                              void *x_out_f16, void *ws, void *stream)
{
    int rc = check_fp_layer(L, B, N);
    if (rc != QUOTA_OK) return rc;
    if (!x_f16 || !pos || !x_out_f16 || !ws) return QUOTA_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const int H = L->H, dh = L->dh, F = L->F, Hkv = L->Hkv > 0 ? L->Hkv : H, d = H * dh, dkv = Hkv * dh;
    const int M = B * N;
    const f16 *x = (const f16 *)x_f16;
    FpWs w = carve_fp(ws, L, B, N);

    fp_rmsnorm_kernel<<<dim3(M), dim3(256), 0, st>>>(x, d, L->gamma1, L->eps, w.h);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    if ((rc = fp_gemm(w.h, M, d, L->wqkv, d + 2 * dkv, nullptr, w.qkv, st)) != QUOTA_OK) return rc;
    const long pairs = (long)M * ((d + 2 * dkv) / 2);
    fp_rope_kernel<<<dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, st>>>(
        w.qkv, M, d, dkv, dh, pos, L->cosT, L->sinT, L->n_pos, w.q, w.k, w.v);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    if ((rc = quota_attention_prefill_gqa(w.q, w.k, w.v, B, N, H, Hkv, dh, 0, 0, w.o, nullptr, nullptr, w.attn,
                                          stream)) != QUOTA_OK)
        return rc;
    if ((rc = fp_gemm(w.o, M, d, L->wo, d, x, w.x1, st)) != QUOTA_OK) return rc;
    fp_rmsnorm_kernel<<<dim3(M), dim3(256), 0, st>>>(w.x1, d, L->gamma2, L->eps, w.h);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    if ((rc = fp_gemm(w.h, M, d, L->wgu, 2 * F, nullptr, w.gu, st)) != QUOTA_OK) return rc;
    const long nz = (long)M * F;
    fp_silu_mul_kernel<<<dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st>>>(w.gu, M, F, w.z);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return fp_gemm(w.z, M, F, L->wdown, d, w.x1, (f16 *)x_out_f16, st);
}

extern "C" int quota_activation_deviation(const void *xq_f16, const void *x_f16, int B, long n_per_sample,
                                          double *diff_norm, double *ref_norm, void *stream)
{
    if (!xq_f16 || !x_f16 || !diff_norm || !ref_norm) return QUOTA_ERR_NULL;
    if (B <= 0 || n_per_sample < 0) return QUOTA_ERR_INVALID_ARG;
    deviation_kernel<<<dim3(B), dim3(1024), 0, (hipStream_t)stream>>>((const f16 *)xq_f16, (const f16 *)x_f16,
                                                                     n_per_sample, diff_norm, ref_norm);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

namespace {
struct ProfileWs {
    f16 *xq, *xf;
    int32_t *pos_out;
    void *rest;
    size_t bytes;
};
ProfileWs carve_profile(void *ws, const quota_layer *Lq, const quota_fp_layer *Lf, int B, int N)
{
    const size_t M = (size_t)B * N, d = (size_t)Lf->H * Lf->dh;
    char *p = (char *)ws;
    ProfileWs w;
    auto take = [&](size_t bytes) { void *r = p; p += up256(bytes); return r; };
    w.xq = (f16 *)take(M * d * 2);
    w.xf = (f16 *)take(M * d * 2);
    w.pos_out = (int32_t *)take(M * 4);
    const size_t a = quota_prefill_workspace_bytes(Lq, B, N), b = quota_fp_block_workspace_bytes(Lf, B, N);
    w.rest = take(a > b ? a : b);           // the two runs are ordered on one stream and share it
    w.bytes = (size_t)(p - (char *)ws);
    return w;
}
}  // namespace

extern "C" size_t quota_profile_block_workspace_bytes(const quota_layer *Lq, const quota_fp_layer *Lf, int B,
                                                      int N)
{
    if (!Lq || check_fp_layer(Lf, B, N) != QUOTA_OK) return 0;
    return carve_profile(nullptr, Lq, Lf, B, N).bytes;
}

extern "C" int quota_profile_block(const quota_layer *Lq, const quota_fp_layer *Lf, const void *x_f16,
                                   const int32_t *pos, int B, int N, quota_kv_cache *scratch_cache,
                                   double *diff_norm, double *ref_norm, void *ws, void *stream)
{
    if (!Lq || !Lf || !x_f16 || !pos || !scratch_cache || !diff_norm || !ref_norm || !ws) return QUOTA_ERR_NULL;
    int rc = check_fp_layer(Lf, B, N);
    if (rc != QUOTA_OK) return rc;
    const int Hkv_q = Lq->Hkv > 0 ? Lq->Hkv : Lq->H, Hkv_f = Lf->Hkv > 0 ? Lf->Hkv : Lf->H;
    if (Lq->H != Lf->H || Lq->dh != Lf->dh || Lq->F != Lf->F || Hkv_q != Hkv_f) return QUOTA_ERR_SHAPE;
    ProfileWs w = carve_profile(ws, Lq, Lf, B, N);

    // the deployed low-bit block, nothing pruned; it validates its own arguments before any launch
    quota_state s;
    s.B = B; s.N = N; s.vis_begin = 0; s.Nv = 0;
    s.x = x_f16; s.pos = pos; s.x_out = w.xq; s.pos_out = w.pos_out;
    quota_score_params p;
    quota_score_params_default(&p);
    const int len0 = scratch_cache->len;
    rc = quota_prefill_layer(Lq, &s, QUOTA_KEEP_ALL, &p, scratch_cache, nullptr, w.rest, stream);
    scratch_cache->len = len0;              // the rows written are scratch: the cache is handed back as it came
    if (rc != QUOTA_OK) return rc;
    if ((rc = quota_fp_block(Lf, x_f16, pos, B, N, w.xf, w.rest, stream)) != QUOTA_OK) return rc;
    return quota_activation_deviation(w.xq, w.xf, B, (long)N * Lf->H * Lf->dh, diff_norm, ref_norm, stream);
}
