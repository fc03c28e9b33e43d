// Decode-side kernels: one new token per sequence attends over the layer's pruned
// 4-bit KV cache (the cache that prefill wrote for retained tokens only), reading the
// codes and group scales straight from HBM and dequantizing them in registers.
// Bandwidth-bound by construction: a step moves H*dh + H*dh/16 bytes per cached token
// and sequence (K and V codes plus fp16 scales), a quarter of an fp16 cache.
#include "common.h"
#include "internal.h"
#include "gemm_common.h"

namespace {

constexpr int DEC_LMAX = QUOTA_MAX_DECODE_ROWS;      // cached rows per sequence the decode calls accept

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

// One workgroup per (sequence, K/V head, RC query heads that share the K/V head), XCD-aware order;
// RC is 1 when every query head has its own K/V head, else 2.  The workgroups of a K/V head are
// neighbours on one XCD, so its rows come from HBM once and from that XCD's L2 afterwards.  The
// cached rows are walked in tiles of DEC_TILE tokens with a running softmax (maximum, sum,
// rescaled output), so the scores of one tile are all the LDS the kernel needs, whatever the
// cache length.
//   loads:   the walk is latency-bound (a workgroup owns a few tens of KB), so every K and V load
//            of a tile is issued before the first use: UN passes of 512 lanes x 16 bytes each;
//   scores:  DH/32 lanes per token, each holds 16 contiguous bytes of the token's K codes (32
//            channels) -- a wave reads whole 64- or 32-byte row segments -- dequantizes them as
//            packed fp16 pairs and dots them with the query; the lanes of a token add up by shuffles;
//   output:  the same lanes own 32 channels of V each and accumulate p * v_hat over their share of
//            the tokens; the token lanes are summed through LDS in a fixed order at the end.
// step_dev (optional): the cache length is len + *step_dev (a HIP-graph-captured decode loop keeps
// its step count on the device).
constexpr int DEC_TILE = 512;
constexpr int DEC_THREADS = 512;     // 8 waves: with two workgroups on a CU every SIMD has four waves to interleave

template <int DH, int RC>
__global__ __launch_bounds__(DEC_THREADS, RC == 1 ? 4 : 2) void decode_attention_kernel(
    const f16 *__restrict__ q, int d, int dkv, int rep, const uint32_t *__restrict__ kc,
    const f16 *__restrict__ ks, const uint32_t *__restrict__ vc, const f16 *__restrict__ vs, int capacity,
    int len, const int32_t *__restrict__ step_dev, int max_steps, f16 *__restrict__ o, int n_kv_heads)
{
    constexpr int PPT = DH / 32;            // 16-byte pieces (lanes) per token and head
    constexpr int TP = DEC_THREADS / PPT;   // tokens per pass of the workgroup
    constexpr int UN = DEC_TILE / TP;       // passes per tile
    constexpr int WPT = DH / 8;             // packed dwords per token and head
    constexpr int GPT = DH / 64;            // scale groups per token and head
    __shared__ h2 qp[RC][DH / 2];           // q as pairs: qp[r][4 i + e] = (q[8 i + e], q[8 i + e + 4])
    __shared__ float sc[RC][DEC_TILE];
    __shared__ float red[32 * (128 + 1)];   // 128 token lanes at a time: [32 channels][128 lanes], padded
    constexpr int NW = DEC_THREADS / 64;    // waves
    constexpr int NQ = DEC_THREADS / 128;   // rounds of the final sum (128 token lanes each)
    __shared__ float wred[2][RC][NW];
    // (sequence, head) pairs are dealt to the 8 XCDs in contiguous ranges: the heads of a sequence
    // share the 128-byte lines of its cache rows (two heads' codes, all heads' scales), and each
    // XCD has its own L2
    const int n_pass = (rep + RC - 1) / RC;            // workgroups per K/V head: RC query heads each
    const int work = xcd_remap(blockIdx.x, gridDim.x);
    const int r0 = (work % n_pass) * RC, h = (work / n_pass) % n_kv_heads, b = work / (n_pass * n_kv_heads);
    const int tid = threadIdx.x, wave = tid >> 6;
    const int piece = tid % PPT, tl = tid / PPT;
    const int wave_t0 = (tid & ~63) / PPT;  // first token of this wave within a pass
    const int n32 = dkv >> 3, ng = dkv >> 6;
    int L = len;
    if (step_dev) L += min(max(*step_dev, 0), max_steps - 1) + 1;      // the row this step appended included
    const float scale = 1.0f / sqrtf((float)DH);
    const size_t row0 = (size_t)b * capacity;

    {
        const int nr = min(RC, rep - r0);
        if (tid < RC * (DH / 2)) {
            const int r = tid / (DH / 2), i = tid % (DH / 2);
            const int hq = min(h * rep + r0 + r, h * rep + rep - 1);
            const f16 *qh = q + (size_t)b * d + hq * DH + 8 * (i >> 2) + (i & 3);
            qp[r][i] = h2{qh[0], qh[4]};
        }
        __syncthreads();
        h2 qr[RC][16];                      // this lane's 32 channels of each query, as pairs
#pragma unroll
        for (int r = 0; r < RC; ++r)
#pragma unroll
            for (int i = 0; i < 16; ++i) qr[r][i] = qp[r][16 * piece + i];
        float m_run[RC], l_run[RC], acc[RC][32];
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            m_run[r] = -INFINITY;
            l_run[r] = 0.0f;
#pragma unroll
            for (int e = 0; e < 32; ++e) acc[r][e] = 0.0f;
        }
        for (int t0 = 0; t0 < L; t0 += DEC_TILE) {
            const int tn = min(DEC_TILE, L - t0);
            uint4 kq[UN], vq[UN];
            _Float16 ksc[UN], vsc[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int t = u * TP + tl;
                const size_t row = row0 + t0 + (t < tn ? t : 0);
                kq[u] = *reinterpret_cast<const uint4 *>(kc + row * n32 + h * WPT + 4 * piece);
                ksc[u] = ks[row * ng + h * GPT + (piece >> 1)];
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int t = u * TP + tl;
                const size_t row = row0 + t0 + (t < tn ? t : 0);
                vq[u] = *reinterpret_cast<const uint4 *>(vc + row * n32 + h * WPT + 4 * piece);
                vsc[u] = vs[row * ng + h * GPT + (piece >> 1)];
            }
            // ---- scores of the tile
            float mx[RC];
#pragma unroll
            for (int r = 0; r < RC; ++r) mx[r] = -INFINITY;
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                if (u * TP + wave_t0 >= tn) continue;       // the whole wave is past the end
                const int t = u * TP + tl;
                const bool ok = t < tn;
                const h2 s2 = h2{ksc[u], ksc[u]};
                const uint32_t ww[4] = {kq[u].x ^ 0x88888888u, kq[u].y ^ 0x88888888u, kq[u].z ^ 0x88888888u,
                                        kq[u].w ^ 0x88888888u};
                float dot[RC][4];           // four independent chains: the dot instruction accumulates in place
#pragma unroll
                for (int r = 0; r < RC; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) dot[r][i] = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {       // channels (8 id + e, 8 id + e + 4), id = 4 piece + i
                        const h2 kh = dequant_pair(ww[i], e, s2);
#pragma unroll
                        for (int r = 0; r < RC; ++r)
                            dot[r][i] = __builtin_amdgcn_fdot2(qr[r][4 * i + e], kh, dot[r][i], false);
                    }
#pragma unroll
                for (int r = 0; r < RC; ++r) {
                    float v = (dot[r][0] + dot[r][1]) + (dot[r][2] + dot[r][3]);
                    v += __shfl_xor(v, 1, 64);
                    if (PPT == 4) v += __shfl_xor(v, 2, 64);
                    v *= scale;
                    if (ok && piece == 0) sc[r][t] = v;
                    if (ok) mx[r] = fmaxf(mx[r], v);
                }
            }
#pragma unroll
            for (int r = 0; r < RC; ++r) {
                mx[r] = wave_max(mx[r]);
                if ((tid & 63) == 0) wred[0][r][wave] = mx[r];
            }
            __syncthreads();                // scores and wave maxima visible
            float alpha[RC], m_new[RC], sum[RC];
#pragma unroll
            for (int r = 0; r < RC; ++r) {
                float tm = wred[0][r][0];
#pragma unroll
                for (int w = 1; w < NW; ++w) tm = fmaxf(tm, wred[0][r][w]);
                m_new[r] = fmaxf(m_run[r], tm);
                alpha[r] = __expf(m_run[r] - m_new[r]);      // 0 on the first tile
                m_run[r] = m_new[r];
                sum[r] = 0.0f;
                for (int t = tid; t < tn; t += DEC_THREADS) {
                    const float p = __expf(sc[r][t] - m_new[r]);
                    sc[r][t] = p;
                    sum[r] += p;
                }
                sum[r] = wave_sum(sum[r]);
                if ((tid & 63) == 0) wred[1][r][wave] = sum[r];
            }
            __syncthreads();                // probabilities and wave sums visible
#pragma unroll
            for (int r = 0; r < RC; ++r) {
                float ts = wred[1][r][0];
#pragma unroll
                for (int w = 1; w < NW; ++w) ts += wred[1][r][w];
                l_run[r] = l_run[r] * alpha[r] + ts;
#pragma unroll
                for (int e = 0; e < 32; ++e) acc[r][e] *= alpha[r];
            }
            // ---- p * v_hat of the tile
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                if (u * TP + wave_t0 >= tn) continue;
                const int t = u * TP + tl;
                const bool ok = t < tn;
                const h2 s2 = h2{vsc[u], vsc[u]};
                const uint32_t ww[4] = {vq[u].x ^ 0x88888888u, vq[u].y ^ 0x88888888u, vq[u].z ^ 0x88888888u,
                                        vq[u].w ^ 0x88888888u};
                float pv[RC];
#pragma unroll
                for (int r = 0; r < RC; ++r) pv[r] = ok ? sc[r][t] : 0.0f;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const h2 vh = dequant_pair(ww[i], e, s2);
#pragma unroll
                        for (int r = 0; r < RC; ++r) {
                            acc[r][8 * i + e] = fmaf(pv[r], (float)vh[0], acc[r][8 * i + e]);
                            acc[r][8 * i + e + 4] = fmaf(pv[r], (float)vh[1], acc[r][8 * i + e + 4]);
                        }
                    }
            }
            __syncthreads();                // the tile's scores have been consumed
        }
        // ---- the token lanes meet in LDS, 128 of them at a time, summed in lane order (red is
        // laid out [channel][token lane] so that the lanes of a wave write consecutive words; the
        // loop over r is unrolled to keep acc in registers)
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            if (r >= nr) break;
            float out = 0.0f;
            for (int round = 0; round < NQ; ++round) {
                __syncthreads();
                if (tl / (TP / NQ) == round) {
#pragma unroll
                    for (int e = 0; e < 32; ++e) red[e * (128 + 1) + (tl % (TP / NQ)) * PPT + piece] = acc[r][e];
                }
                __syncthreads();
                if (tid < DH) {
                    const int pc = tid >> 5, e = tid & 31;
#pragma unroll 4
                    for (int i = 0; i < TP / NQ; ++i) out += red[e * (128 + 1) + i * PPT + pc];
                }
            }
            if (tid < DH) o[(size_t)b * d + (h * rep + r0 + r) * DH + tid] = (f16)(out / l_run[r]);
        }
    }
}

__global__ void advance_step_kernel(int32_t *step) { *step += 1; }

}  // namespace

int quota_internal_advance_step(int32_t *step_dev, hipStream_t st)
{
    advance_step_kernel<<<1, 1, 0, st>>>(step_dev);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" int quota_advance_step(int32_t *step_dev, void *stream)
{
    if (!step_dev) return QUOTA_ERR_NULL;
    return quota_internal_advance_step(step_dev, (hipStream_t)stream);
}

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
    const bool stepped = cache->step_dev != nullptr;     // length = len + *step_dev + 1 (read on the device)
    if (cache->B <= 0 || cache->H <= 0 || Hq <= 0 || cache->len > cache->capacity ||
        (stepped ? cache->len < 0 || cache->max_steps <= 0 || cache->len + cache->max_steps > cache->capacity
                 : cache->len <= 0))
        return QUOTA_ERR_INVALID_ARG;
    const int longest = stepped ? cache->len + cache->max_steps : cache->len;
    if ((cache->dh != 64 && cache->dh != 128) || longest > DEC_LMAX || Hq % cache->H != 0)
        return QUOTA_ERR_SHAPE;
    const int d = Hq * cache->dh, dkv = cache->H * cache->dh, rep = Hq / cache->H;
    hipStream_t st = (hipStream_t)stream;
    const double rows = (double)cache->B * longest;
    ProfScope prof(QUOTA_K_ATTENTION_DECODE, 4.0 * rows * d, rows * (dkv + dkv / 16.0) + 4.0 * cache->B * d, st);
    const int rc = rep == 1 ? 1 : 2;
    dim3 grid(cache->H * cache->B * ((rep + rc - 1) / rc)), block(DEC_THREADS);
    auto kernel = cache->dh == 128 ? (rep == 1 ? decode_attention_kernel<128, 1> : decode_attention_kernel<128, 2>)
                                   : (rep == 1 ? decode_attention_kernel<64, 1> : decode_attention_kernel<64, 2>);
    kernel<<<grid, block, 0, st>>>(
        (const f16 *)q_f16, d, dkv, rep, (const uint32_t *)cache->k_codes, (const f16 *)cache->k_scales,
        (const uint32_t *)cache->v_codes, (const f16 *)cache->v_scales, cache->capacity, cache->len,
        cache->step_dev, cache->max_steps, (f16 *)o_f16, cache->H);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

extern "C" int quota_attention_decode(const void *q_f16, const quota_kv_cache *cache, void *o_f16,
                                      void *stream)
{
    if (!cache) return QUOTA_ERR_NULL;
    return quota_attention_decode_gqa(q_f16, cache->H, cache, o_f16, stream);
}
