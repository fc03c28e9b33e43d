// quota_prefill_layer: host-side sequencing of one W4A4 decoder layer with
// in-layer visual-token pruning.  No device allocation, no synchronisation:
// every intermediate lives in the caller's workspace and every step is a
// kernel enqueued on the caller's stream (safe to capture in a HIP graph).
#include "common.h"
#include "internal.h"

namespace {

// K/V heads of a layer (0 in the descriptor means: as many as query heads)
inline int kv_heads(const quota_layer *L) { return L->Hkv > 0 ? L->Hkv : L->H; }

struct Carver {
    char *base;
    size_t off;
    template <typename T>
    T *take(size_t count)
    {
        size_t bytes = (count * sizeof(T) + 255) & ~(size_t)255;
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += bytes;
        return p;
    }
};

struct LayerWs {
    uint8_t *qa;        // packed int4 activations of the current GEMM input
    float *sa;
    f16 *qkv, *q_rot, *khat, *vhat, *o;
    uint8_t *skc, *svc; // staged 4-bit K/V of all rows
    f16 *sks, *svs;
    float *sumsq, *ressq, *cm_inter, *cm_intra, *score;
    int32_t *keep_idx, *rows;
    f16 *x_keep, *x1, *gu;
    void *attn_ws;
    size_t bytes;
};

LayerWs carve(void *ws, int B, int N, int H, int Hkv, int dh, int F)
{
    Carver c{(char *)ws, 0};
    LayerWs w;
    size_t M = (size_t)B * N, d = (size_t)H * dh, dkv = (size_t)Hkv * dh;
    size_t kmax = d > (size_t)F ? d : (size_t)F;
    w.qa = c.take<uint8_t>(M * kmax / 2);
    w.sa = c.take<float>(M);
    w.qkv = c.take<f16>(M * (d + 2 * dkv));
    w.q_rot = c.take<f16>(M * d);
    w.khat = c.take<f16>(M * dkv);
    w.vhat = c.take<f16>(M * dkv);
    w.o = c.take<f16>(M * d);
    w.skc = c.take<uint8_t>(M * dkv / 2);
    w.svc = c.take<uint8_t>(M * dkv / 2);
    w.sks = c.take<f16>(M * dkv / 64);
    w.svs = c.take<f16>(M * dkv / 64);
    w.sumsq = c.take<float>(M);
    w.ressq = c.take<float>(M);
    w.cm_inter = c.take<float>(M);
    w.cm_intra = c.take<float>(M);
    w.score = c.take<float>(M);
    w.keep_idx = c.take<int32_t>(M);
    w.rows = c.take<int32_t>(M);
    w.x_keep = c.take<f16>(M * d);
    w.x1 = c.take<f16>(M * d);
    w.gu = c.take<f16>(M * 2 * (size_t)F);
    w.attn_ws = c.take<char>(quota_attention_workspace_bytes(B, N, H, dh));
    w.bytes = c.off;
    return w;
}

__global__ void copy_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, long n,
                                int seg, long src_stride, long src_off)
{
    // dst[b*seg + i] = src[b*src_stride + src_off + i]
    long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= n) return;
    long b = t / seg, i = t % seg;
    dst[t] = src[b * src_stride + src_off + i];
}

int dump(void *dst, const void *src, size_t bytes, hipStream_t st)
{
    if (!dst || bytes == 0) return QUOTA_OK;
    return hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st) == hipSuccess ? QUOTA_OK
                                                                                       : QUOTA_ERR_HIP;
}

}  // namespace

#define TRY(expr)                         \
    do {                                  \
        int rc_ = (expr);                 \
        if (rc_ != QUOTA_OK) return rc_;  \
    } while (0)

// QKV projection of the quantized rows in w.qa, RoPE at `pos`, 4-bit K/V of every row: one
// kernel (the GEMM with the fused epilogue) when the shape allows it, else the GEMM followed by
// the stand-alone RoPE/KV kernel.  Both give the same bits.  want_qkv: also keep the plain
// projection output in w.qkv.
static int qkv_rope_kv_quant(const quota_layer *L, const LayerWs &w, int M, const int32_t *pos,
                             bool want_qkv, hipStream_t st, quota_kv_cache *append_to = nullptr)
{
    const int d = L->H * L->dh, Hkv = kv_heads(L), dkv = Hkv * L->dh;
    quota_qkv_epilogue qe;
    qe.pos = pos; qe.cosT = L->cosT; qe.sinT = L->sinT; qe.n_pos = L->n_pos; qe.d = d; qe.dkv = dkv;
    qe.dh = L->dh;
    qe.q_rot = w.q_rot; qe.khat = w.khat; qe.vhat = w.vhat;
    qe.k_codes = (uint32_t *)w.skc; qe.v_codes = (uint32_t *)w.svc;
    qe.k_scales = w.sks; qe.v_scales = w.svs;
    qe.code_row_stride = 1; qe.code_row_offset = 0;
    qe.row_step = nullptr; qe.max_steps = 1;
    if (append_to) {        // decode: row b is sequence b's new token; its K/V go straight to cache row len
        qe.k_codes = (uint32_t *)append_to->k_codes; qe.v_codes = (uint32_t *)append_to->v_codes;
        qe.k_scales = (f16 *)append_to->k_scales; qe.v_scales = (f16 *)append_to->v_scales;
        qe.code_row_stride = append_to->capacity; qe.code_row_offset = append_to->len;
        qe.row_step = append_to->step_dev; qe.max_steps = append_to->max_steps;
    }
    int rc = quota_internal_w4a4_gemm_qkv(w.qa, w.sa, M, &L->qkv, want_qkv ? w.qkv : nullptr, &qe, st);
    if (rc != QUOTA_ERR_SHAPE) return rc;
    if (append_to && append_to->step_dev) return QUOTA_ERR_SHAPE;      // the device-side step needs the fused form
    TRY(quota_w4a4_gemm(w.qa, w.sa, M, &L->qkv, w.qkv, d + 2 * dkv, nullptr, 0, nullptr, st));
    TRY(quota_internal_rope_kv_quant(w.qkv, M, L->H, Hkv, L->dh, pos, L->cosT, L->sinT, L->n_pos, w.q_rot,
                                     w.khat, w.vhat, w.skc, w.sks, w.svc, w.svs, st));
    return append_to ? quota_internal_kv_append_rows(dkv, w.skc, w.sks, w.svc, w.svs, append_to, st) : QUOTA_OK;
}

extern "C" size_t quota_prefill_workspace_bytes(const quota_layer *L, int B, int N)
{
    if (!L || B <= 0 || N <= 0 || L->H <= 0 || L->dh <= 0 || L->F <= 0) return 0;
    return carve(nullptr, B, N, L->H, kv_heads(L), L->dh, L->F).bytes;
}

// Everything a later step of a layer call would reject, checked before the first launch.
static int check_layer(const quota_layer *L, int B, const quota_kv_cache *cache)
{
    if (!L->gamma1 || !L->gamma2 || !L->cosT || !L->sinT) return QUOTA_ERR_NULL;
    if (!cache->k_codes || !cache->k_scales || !cache->v_codes || !cache->v_scales) return QUOTA_ERR_NULL;
    const quota_weights *ws[4] = {&L->qkv, &L->o, &L->gu, &L->down};
    for (const quota_weights *w : ws)
        if (!w->packed || !w->scales) return QUOTA_ERR_NULL;
    const int H = L->H, dh = L->dh, F = L->F;
    if (B <= 0 || H <= 0 || F <= 0 || L->n_pos <= 0 || !(L->eps >= 0.0f) || cache->len < 0 || cache->capacity < 0)
        return QUOTA_ERR_INVALID_ARG;
    const int d = H * dh, Hkv = kv_heads(L), dkv = Hkv * dh;
    if ((dh != 64 && dh != 128) || Hkv <= 0 || H % Hkv != 0 || F % 32 != 0 || d > QUOTA_MAX_MODEL_WIDTH ||
        F > QUOTA_MAX_ROW_COLS || dkv / 64 > 256)
        return QUOTA_ERR_SHAPE;
    if (L->qkv.N != d + 2 * dkv || L->qkv.K != d || L->o.N != d || L->o.K != d || L->gu.N != 2 * F ||
        L->gu.K != d || L->down.N != d || L->down.K != F)
        return QUOTA_ERR_SHAPE;
    for (const quota_weights *w : ws)
        if (w->N % 64 != 0 || w->K % 32 != 0) return QUOTA_ERR_SHAPE;
    if (cache->B != B || cache->H != Hkv || cache->dh != dh) return QUOTA_ERR_SHAPE;
    return QUOTA_OK;
}

extern "C" int quota_prefill_layer(const quota_layer *L, quota_state *s, int K_l,
                                   const quota_score_params *p, quota_kv_cache *cache,
                                   const quota_taps *taps, void *ws, void *stream)
{
    if (!L || !s || !p || !cache || !ws || !s->x || !s->pos || !s->x_out || !s->pos_out) return QUOTA_ERR_NULL;
    const int B = s->B, N = s->N, vb = s->vis_begin, Nv = s->Nv, H = L->H, dh = L->dh, F = L->F;
    TRY(check_layer(L, B, cache));
    if (N <= 0 || vb < 0 || Nv < 0 || vb + Nv > N || K_l < QUOTA_KEEP_ALL) return QUOTA_ERR_INVALID_ARG;
    if (p->pct_lo < 0 || p->pct_hi > 100 || p->pct_lo > p->pct_hi) return QUOTA_ERR_INVALID_ARG;
    const bool candidate = K_l != QUOTA_KEEP_ALL;        // this layer scores and prunes
    if (candidate && Nv > QUOTA_MAX_SCORED_TOKENS) return QUOTA_ERR_SHAPE;
    const int d = H * dh, Hkv = kv_heads(L), dkv = Hkv * dh;
    const int k_keep = !candidate || K_l > Nv ? Nv : K_l;
    const int n_keep = N - Nv + k_keep;
    if (cache->len + n_keep > cache->capacity) return QUOTA_ERR_CAPACITY;

    hipStream_t st = (hipStream_t)stream;
    LayerWs w = carve(ws, B, N, H, Hkv, dh, F);
    const int M = B * N, Mk = B * n_keep;
    static const quota_taps no_taps = {};
    const quota_taps *t = taps ? taps : &no_taps;
    const bool score = candidate && Nv > 0;

    // attention half on every token that entered the layer (the two vector cues of Eq. 6 are side
    // outputs of the first quantizer, taken only where they are used)
    TRY(quota_rmsnorm_quantize_act(s->x, M, d, d, L->gamma1, L->eps, w.qa, w.sa, score ? w.sumsq : nullptr,
                                   score ? w.ressq : nullptr, nullptr, st));
    TRY(qkv_rope_kv_quant(L, w, M, s->pos, t->qkv != nullptr, st));
    TRY(dump(t->qkv, w.qkv, (size_t)M * (d + 2 * dkv) * 2, st));
    TRY(dump(t->q_rot, w.q_rot, (size_t)M * d * 2, st));
    const float *partial = nullptr;     // per-head column masses; their head mean is taken by the score kernel
    TRY(quota_internal_attention(w.q_rot, w.khat, w.vhat, B, N, H, Hkv, dh, vb, Nv, w.o, score, w.attn_ws,
                                 &partial, st));
    TRY(dump(t->o, w.o, (size_t)M * d * 2, st));
    const f16 *o_used = t->inject_o ? (const f16 *)t->inject_o : w.o;
    const bool inject_cm = t->inject_cm_inter && t->inject_cm_intra;

    // Eq. 6-9: cues -> G -> fused score -> top-K_l over the visual tokens (candidate layers only)
    if (score) {
        if (inject_cm) {
            // the library's own cues are still produced for the dump taps
            if (t->cm_inter || t->cm_intra) {
                TRY(quota_internal_score_topk(w.sumsq + vb, w.ressq + vb, N, nullptr, nullptr, partial, H,
                                              w.cm_inter, w.cm_intra, B, Nv, p, w.score, 0, w.keep_idx, st));
            }
            TRY(quota_internal_score_topk(w.sumsq + vb, w.ressq + vb, N, t->inject_cm_inter,
                                          t->inject_cm_intra, nullptr, 0, nullptr, nullptr, B, Nv, p,
                                          w.score, k_keep, w.keep_idx, st));
        } else {
            TRY(quota_internal_score_topk(w.sumsq + vb, w.ressq + vb, N, nullptr, nullptr, partial, H,
                                          w.cm_inter, w.cm_intra, B, Nv, p, w.score, k_keep, w.keep_idx,
                                          st));
        }
        if (t->sumsq || t->ressq) {
            long n = (long)B * Nv;
            dim3 g((unsigned)((n + 255) / 256)), blk(256);
            if (t->sumsq) copy_f32_kernel<<<g, blk, 0, st>>>(w.sumsq, t->sumsq, n, Nv, N, vb);
            if (t->ressq) copy_f32_kernel<<<g, blk, 0, st>>>(w.ressq, t->ressq, n, Nv, N, vb);
            QUOTA_RETURN_IF_LAUNCH_FAILED();
        }
        TRY(dump(t->cm_inter, w.cm_inter, (size_t)B * Nv * 4, st));
        TRY(dump(t->cm_intra, w.cm_intra, (size_t)B * Nv * 4, st));
        TRY(dump(t->score, w.score, (size_t)B * Nv * 4, st));
        TRY(dump(t->keep_idx, w.keep_idx, (size_t)B * k_keep * 4, st));
    }

    // compaction: kept rows of x / pos move on, their 4-bit K/V go to the cache, and the kept
    // attention-output rows leave the gather already quantized for the output projection
    quota_compact_args ca;
    ca.B = B; ca.N = N; ca.vis_begin = vb; ca.Nv = Nv; ca.k_keep = k_keep; ca.n_keep = n_keep;
    ca.d = d; ca.dkv = dkv; ca.keep_idx = score ? w.keep_idx : nullptr; ca.x = s->x; ca.o = o_used; ca.pos = s->pos;
    ca.skc = w.skc; ca.sks = w.sks; ca.svc = w.svc; ca.svs = w.svs;
    ca.x_out = w.x_keep; ca.o_out = nullptr; ca.oq_out = w.qa; ca.os_out = w.sa;
    ca.pos_out = s->pos_out; ca.rows_out = w.rows;
    ca.cache = cache;
    TRY(quota_internal_compact(&ca, st));
    TRY(dump(t->rows, w.rows, (size_t)Mk * 4, st));

    // token-wise rest of the block on the kept rows only
    if (Mk > 0) {
        TRY(quota_w4a4_gemm(w.qa, w.sa, Mk, &L->o, w.x1, d, w.x_keep, d, nullptr, st));
        TRY(dump(t->x1, w.x1, (size_t)Mk * d * 2, st));
        TRY(quota_rmsnorm_quantize_act(w.x1, Mk, d, d, L->gamma2, L->eps, w.qa, w.sa, nullptr,
                                       nullptr, nullptr, st));
        TRY(quota_w4a4_gemm(w.qa, w.sa, Mk, &L->gu, w.gu, 2 * F, nullptr, 0, nullptr, st));
        TRY(dump(t->gu, w.gu, (size_t)Mk * 2 * F * 2, st));
        TRY(quota_silu_mul_quantize_act(w.gu, Mk, F, w.qa, w.sa, t->z, t->inject_z, st));
        TRY(quota_w4a4_gemm(w.qa, w.sa, Mk, &L->down, s->x_out, d, w.x1, d, nullptr, st));
    }
    // the descriptors move only now that every step has been enqueued
    cache->len += n_keep;
    s->N = n_keep;
    s->Nv = k_keep;
    return QUOTA_OK;
}

extern "C" size_t quota_decode_workspace_bytes(const quota_layer *L, int B)
{
    return quota_prefill_workspace_bytes(L, B, 1);
}

extern "C" int quota_decode_layer(const quota_layer *L, const void *x_f16, const int32_t *pos, int B,
                                  quota_kv_cache *cache, void *x_out_f16, const quota_taps *taps,
                                  void *ws, void *stream)
{
    if (!L || !x_f16 || !pos || !cache || !x_out_f16 || !ws) return QUOTA_ERR_NULL;
    TRY(check_layer(L, B, cache));
    const int H = L->H, dh = L->dh, F = L->F, d = H * dh, Hkv = kv_heads(L), dkv = Hkv * dh;
    const bool stepped = cache->step_dev != nullptr;    // the step count lives on the device (captured loops)
    if (stepped && cache->max_steps <= 0) return QUOTA_ERR_INVALID_ARG;
    const int longest = cache->len + (stepped ? cache->max_steps : 1);
    if (longest > cache->capacity) return QUOTA_ERR_CAPACITY;
    if (longest > QUOTA_MAX_DECODE_ROWS) return QUOTA_ERR_SHAPE;
    if (stepped && (d % 128 != 0 || dkv % 128 != 0)) return QUOTA_ERR_SHAPE;   // needs the fused QKV epilogue

    hipStream_t st = (hipStream_t)stream;
    LayerWs w = carve(ws, B, 1, H, Hkv, dh, F);
    static const quota_taps no_taps = {};
    const quota_taps *t = taps ? taps : &no_taps;

    TRY(quota_rmsnorm_quantize_act(x_f16, B, d, d, L->gamma1, L->eps, w.qa, w.sa, nullptr, nullptr,
                                   nullptr, st));
    // the new token's K/V join the cache first (written by the QKV epilogue itself, or by the
    // append kernel on the unfused path); attention then reads all of it in 4-bit form
    TRY(qkv_rope_kv_quant(L, w, B, pos, t->qkv != nullptr, st, cache));
    TRY(dump(t->qkv, w.qkv, (size_t)B * (d + 2 * dkv) * 2, st));
    TRY(dump(t->q_rot, w.q_rot, (size_t)B * d * 2, st));
    quota_kv_cache grown = *cache;      // what the attention reads: the row just written included
    if (!stepped) grown.len += 1;       // (with a device-side step the kernel adds step + 1 itself)
    TRY(quota_attention_decode_gqa(w.q_rot, H, &grown, w.o, st));
    TRY(dump(t->o, w.o, (size_t)B * d * 2, st));
    const f16 *o_used = t->inject_o ? (const f16 *)t->inject_o : w.o;

    TRY(quota_quantize_act(o_used, B, d, d, w.qa, w.sa, nullptr, nullptr, st));
    TRY(quota_w4a4_gemm(w.qa, w.sa, B, &L->o, w.x1, d, x_f16, d, nullptr, st));
    TRY(dump(t->x1, w.x1, (size_t)B * d * 2, st));
    TRY(quota_rmsnorm_quantize_act(w.x1, B, d, d, L->gamma2, L->eps, w.qa, w.sa, nullptr, nullptr,
                                   nullptr, st));
    TRY(quota_w4a4_gemm(w.qa, w.sa, B, &L->gu, w.gu, 2 * F, nullptr, 0, nullptr, st));
    TRY(dump(t->gu, w.gu, (size_t)B * 2 * F * 2, st));
    TRY(quota_silu_mul_quantize_act(w.gu, B, F, w.qa, w.sa, t->z, t->inject_z, st));
    TRY(quota_w4a4_gemm(w.qa, w.sa, B, &L->down, x_out_f16, d, w.x1, d, nullptr, st));
    if (!stepped) cache->len += 1;      // only now that every step has been enqueued
    return QUOTA_OK;
}
