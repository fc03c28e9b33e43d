// Decode-side kernels: one new token per sequence attends over the layer's pruned
// 4-bit KV cache (the cache that prefill wrote for retained tokens only), reading the
// codes and group scales straight from HBM and dequantizing them in registers.
// Bandwidth-bound by construction: a step moves H*dh + H*dh/16 bytes per cached token
// and sequence (K and V codes plus fp16 scales), a quarter of an fp16 cache.
#include "common.h"
#include "internal.h"

namespace {

constexpr int DEC_LMAX = QUOTA_MAX_DECODE_ROWS;      // cached rows one workgroup can softmax over (scores live in LDS)

typedef _Float16 h2 __attribute__((ext_vector_type(2)));

// Dequantizes codes e and e+4 (e = 0..3) of a packed dword to x_hat = fp16(code * s) as a half
// pair.  wx = w ^ 0x88888888 turns each two's-complement nibble c into c + 8 in [0, 15];
// 0x6400 | (c + 8) is the fp16 number 1024 + c + 8, so subtracting 1032 leaves the code exactly,
// and the fp16 multiply rounds code * s once, to nearest -- the value the quantizer defines.
__device__ __forceinline__ h2 dequant_pair(uint32_t wx, int e, h2 s2)
{
    const uint32_t bits = ((wx >> (4 * e)) & 0x000F000Fu) | 0x64006400u;
    h2 c = __builtin_bit_cast(h2, bits);
    c = c - h2{(_Float16)1032.0f, (_Float16)1032.0f};
    return c * s2;
}

// Moves the B freshly quantized K/V rows (staged, dense) to row `len` of each sequence.
__global__ __launch_bounds__(256) void kv_append_rows_kernel(
    int d, const uint32_t *__restrict__ skc, const f16 *__restrict__ sks,
    const uint32_t *__restrict__ svc, const f16 *__restrict__ svs, int capacity, int len,
    uint32_t *__restrict__ ckc, f16 *__restrict__ cks, uint32_t *__restrict__ cvc,
    f16 *__restrict__ cvs)
{
    const int b = blockIdx.x, n32 = d >> 3, ng = d >> 6;
    const size_t crow = (size_t)b * capacity + len;
    for (int i = threadIdx.x; i < n32; i += 256) {
        ckc[crow * n32 + i] = skc[(size_t)b * n32 + i];
        cvc[crow * n32 + i] = svc[(size_t)b * n32 + i];
    }
    for (int i = threadIdx.x; i < ng; i += 256) {
        cks[crow * ng + i] = sks[(size_t)b * ng + i];
        cvs[crow * ng + i] = svs[(size_t)b * ng + i];
    }
}

// One workgroup per (head, sequence).  Pass 1: a thread per cached token computes
// q . k_hat (k_hat = fp16(code * scale), the value the quantizer defines) and the scores
// go to LDS; block max / sum; pass 2: DH/8 threads per token each own 8 channels of V and
// accumulate p_t * v_hat_t over their share of the tokens; the token lanes are then summed
// through LDS in a fixed order.
template <int DH>
__global__ __launch_bounds__(256) void decode_attention_kernel(
    const f16 *__restrict__ q, int d, int dkv, int rep, const uint32_t *__restrict__ kc,
    const f16 *__restrict__ ks, const uint32_t *__restrict__ vc, const f16 *__restrict__ vs, int capacity,
    int L, f16 *__restrict__ o)
{
    constexpr int WPT = DH / 8;             // packed dwords per token and head
    constexpr int GPT = DH / 64;            // scale groups per token and head
    constexpr int TL = 256 / WPT;           // token lanes of pass 2
    __shared__ h2 qp[DH / 2];               // q as pairs: qp[4 i + e] = (q[8 i + e], q[8 i + e + 4])
    __shared__ float sc[DEC_LMAX];
    __shared__ float red[TL * DH];
    __shared__ float wred[8];
    const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int h = hq / rep;                 // K/V head read by query head hq (rep query heads per K/V head)
    const int n32 = dkv >> 3, ng = dkv >> 6;
    if (tid < DH / 2) {
        const f16 *qh = q + (size_t)b * d + hq * DH + 8 * (tid >> 2) + (tid & 3);
        qp[tid] = h2{qh[0], qh[4]};
    }
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)DH);

    float mx = -INFINITY;
    for (int t = tid; t < L; t += 256) {
        const size_t row = (size_t)b * capacity + t;
        const uint32_t *kw = kc + row * n32 + h * WPT;
        const f16 *sp = ks + row * ng + h * GPT;
        float dot = 0.0f;
#pragma unroll
        for (int g = 0; g < GPT; ++g) {
            const _Float16 sh = sp[g];
            const h2 s2 = h2{sh, sh};
#pragma unroll
            for (int w4 = 0; w4 < 2; ++w4) {
                const uint4 pk = *reinterpret_cast<const uint4 *>(kw + 8 * g + 4 * w4);
                const uint32_t ww[4] = {pk.x ^ 0x88888888u, pk.y ^ 0x88888888u, pk.z ^ 0x88888888u,
                                        pk.w ^ 0x88888888u};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int e = 0; e < 4; ++e)     // channels (8i + e, 8i + e + 4) of this 32-channel piece
                        dot = __builtin_amdgcn_fdot2(qp[(64 * g + 32 * w4 + 8 * i) / 2 + e],
                                                     dequant_pair(ww[i], e, s2), dot, false);
            }
        }
        dot *= scale;
        sc[t] = dot;
        mx = fmaxf(mx, dot);
    }
    mx = wave_max(mx);
    if ((tid & 63) == 0) wred[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(wred[0], wred[1]), fmaxf(wred[2], wred[3]));
    float sum = 0.0f;
    for (int t = tid; t < L; t += 256) {
        const float p = __expf(sc[t] - mx);
        sc[t] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    if ((tid & 63) == 0) wred[4 + (tid >> 6)] = sum;
    __syncthreads();                        // also publishes every sc[t]
    const float inv = 1.0f / (((wred[4] + wred[5]) + wred[6]) + wred[7]);

    const int cl = tid % WPT, tl = tid / WPT;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    constexpr int UN = 8;                   // tokens in flight per thread: loads first, then the math
    for (int t0 = tl; t0 < L; t0 += TL * UN) {
        uint32_t w[UN];
        f16 sv[UN];
        float pv[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            const int t = t0 + TL * i;
            const bool ok = t < L;
            const size_t row = (size_t)b * capacity + (ok ? t : 0);
            w[i] = vc[row * n32 + h * WPT + cl];
            sv[i] = vs[row * ng + h * GPT + (cl >> 3)];
            pv[i] = ok ? sc[t] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            const uint32_t wx = w[i] ^ 0x88888888u;
            const h2 s2 = h2{sv[i], sv[i]};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const h2 vh = dequant_pair(wx, e, s2);
                acc[e] = fmaf(pv[i], (float)vh[0], acc[e]);
                acc[e + 4] = fmaf(pv[i], (float)vh[1], acc[e + 4]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[tl * DH + 8 * cl + e] = acc[e];
    __syncthreads();
    if (tid < DH) {
        float v = 0.0f;
#pragma unroll 4
        for (int i = 0; i < TL; ++i) v += red[i * DH + tid];
        o[(size_t)b * d + hq * DH + tid] = (f16)(v * inv);
    }
}

}  // namespace

int quota_internal_kv_append_rows(int d, const uint8_t *skc, const void *sks, const uint8_t *svc,
                                  const void *svs, quota_kv_cache *c, hipStream_t st)
{
    if (c->len + 1 > c->capacity) return QUOTA_ERR_CAPACITY;
    ProfScope prof(QUOTA_K_KV_APPEND_ROWS, 0, 2.0 * c->B * (d + d / 16.0), st);
    kv_append_rows_kernel<<<dim3(c->B), dim3(256), 0, st>>>(
        d, (const uint32_t *)skc, (const f16 *)sks, (const uint32_t *)svc, (const f16 *)svs,
        c->capacity, c->len, (uint32_t *)c->k_codes, (f16 *)c->k_scales, (uint32_t *)c->v_codes,
        (f16 *)c->v_scales);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;         // the caller advances cache->len
}

extern "C" int quota_attention_decode_gqa(const void *q_f16, int Hq, const quota_kv_cache *cache,
                                          void *o_f16, void *stream)
{
    if (!q_f16 || !cache || !o_f16 || !cache->k_codes || !cache->k_scales || !cache->v_codes ||
        !cache->v_scales)
        return QUOTA_ERR_NULL;
    if (cache->B <= 0 || cache->H <= 0 || Hq <= 0 || cache->len <= 0 || cache->len > cache->capacity)
        return QUOTA_ERR_INVALID_ARG;
    if ((cache->dh != 64 && cache->dh != 128) || cache->len > DEC_LMAX || Hq % cache->H != 0)
        return QUOTA_ERR_SHAPE;
    const int d = Hq * cache->dh, dkv = cache->H * cache->dh, rep = Hq / cache->H;
    hipStream_t st = (hipStream_t)stream;
    const double rows = (double)cache->B * cache->len;
    ProfScope prof(QUOTA_K_ATTENTION_DECODE, 4.0 * rows * d, rows * (dkv + dkv / 16.0) + 4.0 * cache->B * d, st);
    dim3 grid(Hq, cache->B), block(256);
    if (cache->dh == 128)
        decode_attention_kernel<128><<<grid, block, 0, st>>>(
            (const f16 *)q_f16, d, dkv, rep, (const uint32_t *)cache->k_codes, (const f16 *)cache->k_scales,
            (const uint32_t *)cache->v_codes, (const f16 *)cache->v_scales, cache->capacity,
            cache->len, (f16 *)o_f16);
    else
        decode_attention_kernel<64><<<grid, block, 0, st>>>(
            (const f16 *)q_f16, d, dkv, rep, (const uint32_t *)cache->k_codes, (const f16 *)cache->k_scales,
            (const uint32_t *)cache->v_codes, (const f16 *)cache->v_scales, cache->capacity,
            cache->len, (f16 *)o_f16);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" int quota_attention_decode(const void *q_f16, const quota_kv_cache *cache, void *o_f16,
                                      void *stream)
{
    if (!cache) return QUOTA_ERR_NULL;
    return quota_attention_decode_gqa(q_f16, cache->H, cache, o_f16, stream);
}
