// RoPE + 4-bit K/V quantization, KV-cache append and the compaction gather.
// All bandwidth-bound: one lane owns 8 consecutive channels (one 16-byte load),
// the 8 lanes of a 64-channel KV group reduce their absmax with three
// xor-shuffles and each lane stores one packed dword of 8 codes.
#include "common.h"
#include "internal.h"
#include "rowquant.h"
#include "ropequant.h"

namespace {

// As many K/V heads as query heads: thread t -> (row, 8-channel chunk c) takes the q, k and v
// chunk at the same c, three independent 16-byte loads in flight per thread.
template <int DH>
__global__ __launch_bounds__(256) void rope_kv_quant_mha_kernel(
    const f16 *__restrict__ qkv, int M, int d, const int32_t *__restrict__ pos, int n_pos,
    const float *__restrict__ cosT, const float *__restrict__ sinT, f16 *__restrict__ q_rot,
    f16 *__restrict__ khat, f16 *__restrict__ vhat, uint32_t *__restrict__ kc,
    f16 *__restrict__ ks, uint32_t *__restrict__ vc, f16 *__restrict__ vs)
{
    constexpr int CPH = DH / 8, HALF = CPH / 2;     // chunks per head, per half head
    const int cpr = d >> 3;                          // chunks per row
    long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= (long)M * cpr) return;
    int row = (int)(t / cpr), c = (int)(t % cpr);
    int cc = c % CPH;
    bool second = cc >= HALF;
    const f16 *base = qkv + (size_t)row * 3 * d + 8 * c;
    Pack16 q, k, v;
    q.u = *reinterpret_cast<const uint4 *>(base);
    k.u = *reinterpret_cast<const uint4 *>(base + d);
    v.u = *reinterpret_cast<const uint4 *>(base + 2 * d);
    Pack16 qp, kp;                                   // rotate-half partner chunk
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        qp.w[i] = __shfl_xor(q.w[i], HALF, 64);
        kp.w[i] = __shfl_xor(k.w[i], HALF, 64);
    }
    const int pr = min(max(pos[row], 0), n_pos - 1);     // never index outside the tables
    const float *cp = cosT + (size_t)pr * (DH / 2) + 8 * (cc % HALF);
    const float *sp = sinT + (size_t)pr * (DH / 2) + 8 * (cc % HALF);
    float cs[8], sn[8];
    *reinterpret_cast<float4 *>(cs) = *reinterpret_cast<const float4 *>(cp);
    *reinterpret_cast<float4 *>(cs + 4) = *reinterpret_cast<const float4 *>(cp + 4);
    *reinterpret_cast<float4 *>(sn) = *reinterpret_cast<const float4 *>(sp);
    *reinterpret_cast<float4 *>(sn + 4) = *reinterpret_cast<const float4 *>(sp + 4);
    Pack16 qo, ko;
    float kf[8], vf[8];
    rope8(q, qp, cs, sn, second, qo);
    rope8(k, kp, cs, sn, second, ko);            // rotated k is an fp16 tensor
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        kf[e] = (float)ko.h[e];
        vf[e] = (float)v.h[e];
    }
    *reinterpret_cast<uint4 *>(q_rot + (size_t)row * d + 8 * c) = qo.u;
    Pack16 kh, vh;
    f16 ksc, vsc;
    uint32_t kw = kv_quant8(kf, &ksc, &kh);
    uint32_t vw = kv_quant8(vf, &vsc, &vh);
    *reinterpret_cast<uint4 *>(khat + (size_t)row * d + 8 * c) = kh.u;
    *reinterpret_cast<uint4 *>(vhat + (size_t)row * d + 8 * c) = vh.u;
    kc[(size_t)row * cpr + c] = kw;
    vc[(size_t)row * cpr + c] = vw;
    if ((c & 7) == 0) {
        ks[(size_t)row * (cpr >> 3) + (c >> 3)] = ksc;
        vs[(size_t)row * (cpr >> 3) + (c >> 3)] = vsc;
    }
}

// thread t -> (row, 8-channel chunk c of the q | k | v row).  q has d = H*dh channels, k and v
// dkv = Hkv*dh each (dkv = d unless K/V heads are shared by groups of query heads).
template <int DH>
__global__ __launch_bounds__(256) void rope_kv_quant_kernel(
    const f16 *__restrict__ qkv, int M, int d, int dkv, const int32_t *__restrict__ pos, int n_pos,
    const float *__restrict__ cosT, const float *__restrict__ sinT, f16 *__restrict__ q_rot,
    f16 *__restrict__ khat, f16 *__restrict__ vhat, uint32_t *__restrict__ kc,
    f16 *__restrict__ ks, uint32_t *__restrict__ vc, f16 *__restrict__ vs)
{
    constexpr int CPH = DH / 8, HALF = CPH / 2;     // chunks per head, per half head
    const int cq = d >> 3, ckv = dkv >> 3, cpr = cq + 2 * ckv;      // chunks: q part, k or v part, row
    long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= (long)M * cpr) return;
    const int row = (int)(t / cpr), c = (int)(t % cpr);
    // region boundaries are multiples of a head (16 or 8 chunks), so the 8 lanes of a KV group
    // and the two halves of a head always sit in the same region
    const int region = c < cq ? 0 : (c < cq + ckv ? 1 : 2);
    const int cr = c - (region == 0 ? 0 : (region == 1 ? cq : cq + ckv));      // chunk inside the region
    const int cc = cr % CPH;
    const bool second = cc >= HALF;
    Pack16 x, xp, xo;
    x.u = *reinterpret_cast<const uint4 *>(qkv + (size_t)row * (d + 2 * dkv) + 8 * c);
    if (region < 2) {
#pragma unroll
        for (int i = 0; i < 4; ++i) xp.w[i] = __shfl_xor(x.w[i], HALF, 64);     // rotate-half partner chunk
        const int pr = min(max(pos[row], 0), n_pos - 1);     // never index outside the tables
        const float *cp = cosT + (size_t)pr * (DH / 2) + 8 * (cc % HALF);
        const float *sp = sinT + (size_t)pr * (DH / 2) + 8 * (cc % HALF);
        float cs[8], sn[8];
        *reinterpret_cast<float4 *>(cs) = *reinterpret_cast<const float4 *>(cp);
        *reinterpret_cast<float4 *>(cs + 4) = *reinterpret_cast<const float4 *>(cp + 4);
        *reinterpret_cast<float4 *>(sn) = *reinterpret_cast<const float4 *>(sp);
        *reinterpret_cast<float4 *>(sn + 4) = *reinterpret_cast<const float4 *>(sp + 4);
        rope8(x, xp, cs, sn, second, xo);            // rotated q / k are fp16 tensors
    } else {
        xo = x;
    }
    if (region == 0) {
        *reinterpret_cast<uint4 *>(q_rot + (size_t)row * d + 8 * cr) = xo.u;
        return;
    }
    float f[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (float)xo.h[e];
    Pack16 hat;
    f16 sc;
    const uint32_t word = kv_quant8(f, &sc, &hat);
    f16 *xh = region == 1 ? khat : vhat;
    uint32_t *codes = region == 1 ? kc : vc;
    f16 *scales = region == 1 ? ks : vs;
    *reinterpret_cast<uint4 *>(xh + (size_t)row * dkv + 8 * cr) = hat.u;
    codes[(size_t)row * ckv + cr] = word;
    if ((cr & 7) == 0) scales[(size_t)row * (ckv >> 3) + (cr >> 3)] = sc;
}

__global__ __launch_bounds__(256) void kv_quant_append_kernel(
    const f16 *__restrict__ k, const f16 *__restrict__ v, int B, int N, int d,
    const int32_t *__restrict__ keep_rows, int n_keep, int capacity, int len,
    uint32_t *__restrict__ kc, f16 *__restrict__ ks, uint32_t *__restrict__ vc, f16 *__restrict__ vs)
{
    const int cpr = d >> 3;
    long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= (long)B * n_keep * cpr) return;
    int c = (int)(t % cpr);
    long rj = t / cpr;
    int j = (int)(rj % n_keep), b = (int)(rj / n_keep);
    int src = keep_rows ? keep_rows[(size_t)b * n_keep + j] : j;
    src = min(max(src, 0), N - 1);                      // never read outside the sequence
    size_t srow = (size_t)b * N + src, drow = (size_t)b * capacity + len + j;
    Pack16 kk, vv;
    kk.u = *reinterpret_cast<const uint4 *>(k + srow * d + 8 * c);
    vv.u = *reinterpret_cast<const uint4 *>(v + srow * d + 8 * c);
    float kf[8], vf[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { kf[e] = (float)kk.h[e]; vf[e] = (float)vv.h[e]; }
    f16 ksc, vsc;
    uint32_t kw = kv_quant8(kf, &ksc, nullptr);
    uint32_t vw = kv_quant8(vf, &vsc, nullptr);
    kc[drow * cpr + c] = kw;
    vc[drow * cpr + c] = vw;
    if ((c & 7) == 0) {
        ks[drow * (cpr >> 3) + (c >> 3)] = ksc;
        vs[drow * (cpr >> 3) + (c >> 3)] = vsc;
    }
}

// Compaction gather of the layer (one workgroup per kept row): copies the
// kept rows of the hidden state and the positions, moves their staged 4-bit
// K/V rows into the layer's cache, and gathers the attention-output row --
// copied (o_out) and/or quantized for the output projection (oq_out, os_out).
// NCH = 16-byte chunks of a row per thread (2 covers 4096 columns, 8 covers 16384).  All loads
// of a thread that do not depend on each other are issued together (unconditional, at clamped
// indices): after the one dependent step -- the kept index, then the rows it names -- the kernel
// needs a single memory round trip.
template <int NCH>
__global__ __launch_bounds__(256) void compact_rows_kernel(
    int N, int vis_begin, int Nv, int k_keep, int n_keep, const int32_t *__restrict__ keep_idx,
    int d, int dkv, const f16 *__restrict__ x, const f16 *__restrict__ o, const int32_t *__restrict__ pos,
    const uint32_t *__restrict__ skc, const f16 *__restrict__ sks, const uint32_t *__restrict__ svc,
    const f16 *__restrict__ svs, f16 *__restrict__ x_out, f16 *__restrict__ o_out,
    uint32_t *__restrict__ oq_out, float *__restrict__ os_out,
    int32_t *__restrict__ pos_out, int32_t *__restrict__ rows_out, int capacity, int len,
    uint32_t *__restrict__ ckc, f16 *__restrict__ cks, uint32_t *__restrict__ cvc,
    f16 *__restrict__ cvs)
{
    const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    int src;
    if (j < vis_begin) src = j;
    else if (j < vis_begin + k_keep) src = vis_begin + (keep_idx ? keep_idx[(size_t)b * k_keep + (j - vis_begin)] : j - vis_begin);
    else src = j - k_keep + Nv;
    src = min(max(src, 0), N - 1);
    const size_t srow = (size_t)b * N + src, drow = (size_t)b * n_keep + j;
    const size_t crow = (size_t)b * capacity + len + j;
    const int n16 = d >> 3;       // 16-byte pieces in an fp16 row
    const int nkv = dkv >> 3;     // dwords of codes per K or V row (<= n16)
    const int ng = dkv >> 6;      // group scales per K or V row
    const uint4 *xs = reinterpret_cast<const uint4 *>(x + srow * d);
    const uint4 *os = reinterpret_cast<const uint4 *>(o + srow * d);
    const bool want_o = o_out || oq_out;
    __shared__ double sm[12];
    uint4 xv[NCH];
    Pack16 v[NCH];
    uint32_t kw[NCH], vw[NCH];
#pragma unroll
    for (int r = 0; r < NCH; ++r) {
        const int i = tid + ROW_THREADS * r;
        xv[r] = xs[min(i, n16 - 1)];
        if (want_o) v[r].u = os[min(i, n16 - 1)];
        kw[r] = skc[srow * nkv + min(i, nkv - 1)];
        vw[r] = svc[srow * nkv + min(i, nkv - 1)];
    }
    const f16 ksv = sks[srow * ng + min(tid, ng - 1)], vsv = svs[srow * ng + min(tid, ng - 1)];
    const int32_t pv = pos[srow];

    // the attention-output row is copied and/or fed to the activation quantizer in front of the
    // output projection (same code path as the stand-alone quantizer)
    float a = 0.0f;
#pragma unroll
    for (int r = 0; r < NCH; ++r) {
        const int i = tid + ROW_THREADS * r;
        if (i < n16) {
            if (x_out) reinterpret_cast<uint4 *>(x_out + drow * d)[i] = xv[r];
            if (o_out) reinterpret_cast<uint4 *>(o_out + drow * d)[i] = v[r].u;
            if (want_o) {
#pragma unroll
                for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf((float)v[r].h[e]));
            }
        }
        if (i < nkv) {
            ckc[crow * nkv + i] = kw[r];
            cvc[crow * nkv + i] = vw[r];
        }
    }
    if (tid < ng) {
        cks[crow * ng + tid] = ksv;
        cvs[crow * ng + tid] = vsv;
    }
    if (tid == 0) {
        pos_out[drow] = pv;
        if (rows_out) rows_out[drow] = src;
    }
    if (oq_out) {
        double z0 = 0.0, z1 = 0.0;
        block_max_sum2<4>(a, z0, z1, sm);
        float s;
        quantize_cached_row<false, ROW_THREADS, NCH>(v, n16, tid, a, oq_out + drow * n16, s);
        if (tid == 0) os_out[drow] = s;
    }
}

}  // namespace

int quota_internal_compact(const quota_compact_args *a, hipStream_t st)
{
    quota_kv_cache *c = a->cache;
    if (c->len + a->n_keep > c->capacity) return QUOTA_ERR_CAPACITY;
    if (a->d % 8 != 0 || a->d > 8 * ROW_THREADS * 8 || a->dkv > a->d || a->dkv < 64 ||
        a->dkv / 64 > ROW_THREADS)
        return QUOTA_ERR_SHAPE;
    if (a->n_keep == 0) return QUOTA_OK;
    const double rows = (double)a->n_keep * a->B, dd = a->d, dk = a->dkv;
    ProfScope prof(QUOTA_K_COMPACT_ROWS, 0, rows * (2 * (4 * dd + dk + dk / 16) + 8), st);
    auto kernel = a->d <= 4096 ? compact_rows_kernel<2> : compact_rows_kernel<8>;
    kernel<<<dim3(a->n_keep, a->B), dim3(256), 0, st>>>(
        a->N, a->vis_begin, a->Nv, a->k_keep, a->n_keep, a->keep_idx, a->d, a->dkv, (const f16 *)a->x,
        (const f16 *)a->o, a->pos, (const uint32_t *)a->skc, (const f16 *)a->sks,
        (const uint32_t *)a->svc, (const f16 *)a->svs, (f16 *)a->x_out, (f16 *)a->o_out, (uint32_t *)a->oq_out, a->os_out, a->pos_out,
        a->rows_out, c->capacity, c->len, (uint32_t *)c->k_codes, (f16 *)c->k_scales,
        (uint32_t *)c->v_codes, (f16 *)c->v_scales);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;         // the caller advances cache->len once the whole layer is enqueued
}

int quota_internal_rope_kv_quant(const void *qkv_f16, int M, int H, int Hkv, int dh, const int32_t *pos,
                                 const float *cosT, const float *sinT, int n_pos, void *q_rot_f16,
                                 void *khat_f16, void *vhat_f16, uint8_t *k_codes, void *k_scales,
                                 uint8_t *v_codes, void *v_scales, hipStream_t st)
{
    if (!qkv_f16 || !pos || !cosT || !sinT || !q_rot_f16 || !khat_f16 || !vhat_f16 || !k_codes ||
        !k_scales || !v_codes || !v_scales)
        return QUOTA_ERR_NULL;
    if (M < 0 || H <= 0 || Hkv <= 0 || n_pos <= 0) return QUOTA_ERR_INVALID_ARG;
    if ((dh != 64 && dh != 128) || H % Hkv != 0) return QUOTA_ERR_SHAPE;
    if (M == 0) return QUOTA_OK;
    const int d = H * dh, dkv = Hkv * dh;
    long total = Hkv == H ? (long)M * (d >> 3) : (long)M * ((d + 2 * dkv) >> 3);
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    ProfScope prof(QUOTA_K_ROPE_KV_QUANT, 0,
                   (double)M * (2.0 * (d + 2 * dkv) + 2.0 * d + dkv * (4 + 1 + 1.0 / 16)) + 4.0 * M, st);
    if (Hkv == H) {
        if (dh == 128)
            rope_kv_quant_mha_kernel<128><<<grid, block, 0, st>>>(
                (const f16 *)qkv_f16, M, d, pos, n_pos, cosT, sinT, (f16 *)q_rot_f16, (f16 *)khat_f16,
                (f16 *)vhat_f16, (uint32_t *)k_codes, (f16 *)k_scales, (uint32_t *)v_codes, (f16 *)v_scales);
        else
            rope_kv_quant_mha_kernel<64><<<grid, block, 0, st>>>(
                (const f16 *)qkv_f16, M, d, pos, n_pos, cosT, sinT, (f16 *)q_rot_f16, (f16 *)khat_f16,
                (f16 *)vhat_f16, (uint32_t *)k_codes, (f16 *)k_scales, (uint32_t *)v_codes, (f16 *)v_scales);
    } else if (dh == 128)
        rope_kv_quant_kernel<128><<<grid, block, 0, st>>>(
            (const f16 *)qkv_f16, M, d, dkv, pos, n_pos, cosT, sinT, (f16 *)q_rot_f16, (f16 *)khat_f16,
            (f16 *)vhat_f16, (uint32_t *)k_codes, (f16 *)k_scales, (uint32_t *)v_codes,
            (f16 *)v_scales);
    else
        rope_kv_quant_kernel<64><<<grid, block, 0, st>>>(
            (const f16 *)qkv_f16, M, d, dkv, pos, n_pos, cosT, sinT, (f16 *)q_rot_f16, (f16 *)khat_f16,
            (f16 *)vhat_f16, (uint32_t *)k_codes, (f16 *)k_scales, (uint32_t *)v_codes,
            (f16 *)v_scales);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" int quota_rope_kv_quant(const void *qkv_f16, int M, int H, int dh, const int32_t *pos,
                                   const float *cosT, const float *sinT, int n_pos,
                                   void *q_rot_f16, void *khat_f16, void *vhat_f16,
                                   uint8_t *k_codes, void *k_scales, uint8_t *v_codes,
                                   void *v_scales, void *stream)
{
    return quota_internal_rope_kv_quant(qkv_f16, M, H, H, dh, pos, cosT, sinT, n_pos, q_rot_f16, khat_f16,
                                        vhat_f16, k_codes, k_scales, v_codes, v_scales, (hipStream_t)stream);
}

extern "C" int quota_kv_quant_append(const void *k_f16, const void *v_f16, int B, int N, int H,
                                     int dh, const int32_t *keep_rows, int n_keep,
                                     quota_kv_cache *cache, void *stream)
{
    if (!k_f16 || !v_f16 || !cache || !cache->k_codes || !cache->k_scales || !cache->v_codes ||
        !cache->v_scales)
        return QUOTA_ERR_NULL;
    if (B <= 0 || N < 0 || H <= 0 || n_keep < 0 || cache->len < 0) return QUOTA_ERR_INVALID_ARG;
    if (dh % 64 != 0 || cache->H != H || cache->dh != dh || cache->B != B) return QUOTA_ERR_SHAPE;
    if (!keep_rows && n_keep > N) return QUOTA_ERR_INVALID_ARG;
    if (cache->len + n_keep > cache->capacity) return QUOTA_ERR_CAPACITY;
    if (n_keep == 0) return QUOTA_OK;
    int d = H * dh;
    long total = (long)B * n_keep * (d >> 3);
    ProfScope prof(QUOTA_K_KV_QUANT_APPEND, 0, (double)B * n_keep * d * (4 + 1 + 1.0 / 16),
                   (hipStream_t)stream);
    kv_quant_append_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                             (hipStream_t)stream>>>(
        (const f16 *)k_f16, (const f16 *)v_f16, B, N, d, keep_rows, n_keep, cache->capacity,
        cache->len, (uint32_t *)cache->k_codes, (f16 *)cache->k_scales,
        (uint32_t *)cache->v_codes, (f16 *)cache->v_scales);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    cache->len += n_keep;
    return QUOTA_OK;
}
