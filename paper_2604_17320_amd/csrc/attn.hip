// Causal prefill attention over the dequantized 4-bit K/V (fp16 MFMA, fp32
// online softmax) and the attention-cue pass of Eq. 6 (column masses).
//
// Pass 1 works on transposed tiles so that every softmax statistic is a
// per-lane scalar: S^T = K Q^T puts the query on the lane (column) and the
// keys on the accumulator registers; the probabilities then feed
// O^T += V^T P^T straight from those registers (their register->key mapping is
// the k-slot mapping chosen for the B operand of v_mfma_f32_32x32x16_f16; a
// contraction does not care which element sits in which k-slot as long as both
// operands agree, so V^T is read with the same key-to-slot mapping).
//
// Pass 2 owns key columns instead: S = Q K^T puts the key on the lane, so the
// column sums over queries are in-lane adds in a fixed order (deterministic,
// no atomics).  It needs the final log-sum-exp of every query row from pass 1.
#include "common.h"
#include "internal.h"

namespace {

constexpr int KT = 64;       // keys per tile (pass 1), queries per tile (pass 2)

// 2^x on the transcendental unit, without the range handling of exp2f (its extra instructions only
// matter for results below the smallest normal number, which are zero for a softmax anyway)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int DH>
struct AttnSmem {
    alignas(16) f16 k[KT][DH + 8];       // row stride = odd number of 16-byte units: conflict-free 16-byte reads
    alignas(16) f16 vt[DH][KT + 4];      // V transposed: [channel][key]
};

template <int DH>
__global__ __launch_bounds__(256) void attn_fwd_kernel(
    const f16 *__restrict__ q, const f16 *__restrict__ khat, const f16 *__restrict__ vhat, int N,
    int H, int Hkv, f16 *__restrict__ o, float *__restrict__ lse2, float scale_log2)
{
    constexpr int T = DH / 16;       // k-steps (16 channels each) of the QK product
    constexpr int DB = DH / 32;      // 32-channel blocks of the output
    constexpr int CPR = DH / 8;      // 16-byte chunks per head row
    __shared__ AttnSmem<DH> sm;
    const int d = H * DH;
    const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * 128;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hl = lane >> 5;
    const int qw0 = q0 + wave * 32, qi = qw0 + l32;       // this lane's query
    const size_t base = (size_t)b * N * d + (size_t)h * DH;
    // K/V rows have Hkv heads; query head h reads K/V head h / (H / Hkv)
    const int dkv = Hkv * DH;
    const size_t kvbase = (size_t)b * N * dkv + (size_t)(h / (H / Hkv)) * DH;

    f16x8 qf[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        if (qi < N)
            qf[t] = *reinterpret_cast<const f16x8 *>(q + base + (size_t)qi * d + 16 * t + 8 * hl);
        else
            qf[t] = f16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    f32x16 oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    const int q_last_wg = min(q0 + 127, N - 1);
    // Each thread stages 4 + 4 sixteen-byte pieces of a 64-key tile.  The pieces of the
    // NEXT tile are fetched into registers before the current tile is consumed, so the
    // global-memory latency overlaps the MFMAs instead of preceding them.
    constexpr int PER = KT * CPR / 256;
    Pack16 rk[PER], rv[PER];
    auto fetch = [&](int kt0) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = tid + 256 * j;
            const int keyk = i / CPR, ck = i % CPR, keyv = i % KT, cv = i / KT;
            rk[j].u = make_uint4(0, 0, 0, 0);
            rv[j].u = make_uint4(0, 0, 0, 0);
            if (kt0 + keyk < N)
                rk[j].u = *reinterpret_cast<const uint4 *>(khat + kvbase + (size_t)(kt0 + keyk) * dkv + 8 * ck);
            if (kt0 + keyv < N)
                rv[j].u = *reinterpret_cast<const uint4 *>(vhat + kvbase + (size_t)(kt0 + keyv) * dkv + 8 * cv);
        }
    };
    fetch(0);
    for (int kt0 = 0; kt0 <= q_last_wg; kt0 += KT) {
        __syncthreads();
        // K rows (16-byte stores) and V transposed (2-byte stores, lane = key)
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = tid + 256 * j;
            const int keyk = i / CPR, ck = i % CPR, keyv = i % KT, cv = i / KT;
            *reinterpret_cast<uint4 *>(&sm.k[keyk][8 * ck]) = rk[j].u;
#pragma unroll
            for (int e = 0; e < 8; ++e) sm.vt[8 * cv + e][keyv] = rv[j].h[e];
        }
        __syncthreads();
        if (kt0 + KT <= q_last_wg) fetch(kt0 + KT);
        if (kt0 > qw0 + 31) continue;        // tile entirely above this wave's diagonal

        f32x16 s[2];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[sb][r] = 0.0f;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                f16x8 kf = *reinterpret_cast<const f16x8 *>(&sm.k[32 * sb + l32][16 * t + 8 * hl]);
                s[sb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[t], s[sb], 0, 0, 0);
            }
        }
        // the maximum is taken on the raw logits (the scale is positive) and the scale is folded into
        // the exponent's fused multiply-add: exp2(s * scale - m), one instruction per score less
        float mx = -INFINITY;
        // only a tile that reaches this wave's diagonal or the end of the sequence needs the mask
        if (kt0 + KT - 1 > qw0 || kt0 + KT > N) {
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int key = kt0 + 32 * sb + 8 * (r >> 2) + 4 * hl + (r & 3);
                    float v = (key <= qi && key < N) ? s[sb][r] : -INFINITY;
                    s[sb][r] = v;
                    mx = fmaxf(mx, v);
                }
        } else {
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float m_new = fmaxf(m_run, mx * scale_log2);
        float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        float psum = 0.0f;
        // k-slot j of step u holds key 32 sb + 16 u + 8 (j / 4) + 4 hl + j % 4: registers 8u .. 8u+7
        f16x8 pf[2][2];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float p[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) p[j] = fast_exp2(__builtin_fmaf(s[sb][8 * u + j], scale_log2, -m_new));
                psum += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
                pf[sb][u] = f16x8{(f16)p[0], (f16)p[1], (f16)p[2], (f16)p[3],
                                  (f16)p[4], (f16)p[5], (f16)p[6], (f16)p[7]};
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int i = 0; i < DB; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const f16 *vrow = &sm.vt[32 * i + l32][32 * sb + 16 * u + 4 * hl];
                    f16x4 v0 = *reinterpret_cast<const f16x4 *>(vrow);
                    f16x4 v1 = *reinterpret_cast<const f16x4 *>(vrow + 8);
                    f16x8 vf = f16x8{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                    oacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[sb][u], oacc[i], 0, 0, 0);
                }
        }
    }
    float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (qi < N) {
        float inv = 1.0f / l_tot;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f16x4 ov = f16x4{(f16)(oacc[i][4 * g + 0] * inv), (f16)(oacc[i][4 * g + 1] * inv),
                                 (f16)(oacc[i][4 * g + 2] * inv), (f16)(oacc[i][4 * g + 3] * inv)};
                *reinterpret_cast<f16x4 *>(o + base + (size_t)qi * d + 32 * i + 8 * g + 4 * hl) = ov;
            }
        if (hl == 0) lse2[((size_t)b * H + h) * N + qi] = m_run + log2f(l_tot);
    }
}

template <int DH>
struct CmSmem {
    alignas(16) f16 q[KT][DH + 8];
    float lse[KT];
};

// grid: (ceil(Nv/128), H, B); wave w owns the 32 visual keys kb .. kb+31
template <int DH>
__global__ __launch_bounds__(256) void colmass_kernel(
    const f16 *__restrict__ q, const f16 *__restrict__ khat, const float *__restrict__ lse2, int N,
    int H, int Hkv, int vis_begin, int Nv, float *__restrict__ partial, float scale_log2)
{
    constexpr int T = DH / 16, CPR = DH / 8;
    __shared__ CmSmem<DH> sm;
    const int d = H * DH;
    const int b = blockIdx.z, h = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hl = lane >> 5;
    const int kwg = vis_begin + blockIdx.x * 128;         // first key of the workgroup
    const int key = kwg + wave * 32 + l32;                // this lane's key column
    const bool key_ok = key < vis_begin + Nv;
    const size_t base = (size_t)b * N * d + (size_t)h * DH;

    f16x8 kf[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        if (key_ok)
            kf[t] = *reinterpret_cast<const f16x8 *>(khat + (size_t)b * N * (Hkv * DH) + (size_t)(h / (H / Hkv)) * DH +
                                                     (size_t)key * (Hkv * DH) + 16 * t + 8 * hl);
        else
            kf[t] = f16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    float acc_txt = 0.0f, acc_vis = 0.0f;
    constexpr int PER = KT * CPR / 256;
    Pack16 rq[PER];
    float rl = 0.0f;
    auto fetch = [&](int qt0) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = tid + 256 * j, r = i / CPR, c = i % CPR;
            rq[j].u = make_uint4(0, 0, 0, 0);
            if (qt0 + r < N)
                rq[j].u = *reinterpret_cast<const uint4 *>(q + base + (size_t)(qt0 + r) * d + 8 * c);
        }
        if (tid < KT) rl = qt0 + tid < N ? lse2[((size_t)b * H + h) * N + qt0 + tid] : 0.0f;
    };
    const int qt_first = (kwg / KT) * KT;
    fetch(qt_first);
    for (int qt0 = qt_first; qt0 < N; qt0 += KT) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = tid + 256 * j, r = i / CPR, c = i % CPR;
            *reinterpret_cast<uint4 *>(&sm.q[r][8 * c]) = rq[j].u;
        }
        if (tid < KT) sm.lse[tid] = rl;
        __syncthreads();
        if (qt0 + KT < N) fetch(qt0 + KT);
        if (qt0 + KT - 1 < kwg + wave * 32) continue;     // all queries before this wave's keys
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.0f;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                f16x8 qf = *reinterpret_cast<const f16x8 *>(&sm.q[32 * sb + l32][16 * t + 8 * hl]);
                s = __builtin_amdgcn_mfma_f32_32x32x16_f16(qf, kf[t], s, 0, 0, 0);
            }
            // the causal / end-of-sequence mask is only needed when the query block reaches this
            // wave's keys or the end of the sequence (lanes without a key accumulate values that
            // are never stored)
            const int qb0 = qt0 + 32 * sb;
            if (qb0 < kwg + wave * 32 + 31 || qb0 + 32 > N) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int ql = 32 * sb + 8 * (r >> 2) + 4 * hl + (r & 3);
                    int qi = qt0 + ql;
                    float p = fast_exp2(__builtin_fmaf(s[r], scale_log2, -sm.lse[ql]));
                    p = (key <= qi && qi < N) ? p : 0.0f;
                    bool vis = qi >= vis_begin && qi < vis_begin + Nv;
                    acc_vis += vis ? p : 0.0f;
                    acc_txt += vis ? 0.0f : p;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int ql = 32 * sb + 8 * (r >> 2) + 4 * hl + (r & 3);
                    int qi = qt0 + ql;
                    float p = fast_exp2(__builtin_fmaf(s[r], scale_log2, -sm.lse[ql]));
                    bool vis = qi >= vis_begin && qi < vis_begin + Nv;
                    acc_vis += vis ? p : 0.0f;
                    acc_txt += vis ? 0.0f : p;
                }
            }
        }
    }
    acc_txt += __shfl_xor(acc_txt, 32, 64);
    acc_vis += __shfl_xor(acc_vis, 32, 64);
    if (key_ok && hl == 0) {
        size_t oidx = (((size_t)b * H + h) * Nv + (key - vis_begin)) * 2;
        partial[oidx] = acc_txt;
        partial[oidx + 1] = acc_vis;
    }
}

// head mean in head order: cm[b][i] = (1/H) * sum_h partial[b][h][i]
__global__ __launch_bounds__(256) void colmass_reduce_kernel(
    const float *__restrict__ partial, int B, int H, int Nv, float *__restrict__ cm_inter,
    float *__restrict__ cm_intra)
{
    int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= B * Nv) return;
    int b = t / Nv, i = t % Nv;
    float st = 0.0f, sv = 0.0f;
    for (int h = 0; h < H; ++h) {
        size_t idx = (((size_t)b * H + h) * Nv + i) * 2;
        st += partial[idx];
        sv += partial[idx + 1];
    }
    float invH = 1.0f / (float)H;
    if (cm_inter) cm_inter[t] = st * invH;
    if (cm_intra) cm_intra[t] = sv * invH;
}

}  // namespace

extern "C" size_t quota_attention_workspace_bytes(int B, int N, int H, int dh)
{
    (void)dh;
    if (B <= 0 || N <= 0 || H <= 0) return 0;
    // row log-sum-exp [B][H][N] + per-head column masses [B][H][N][2]
    return (size_t)B * H * N * sizeof(float) * 3;
}

int quota_internal_attention(const void *q_f16, const void *khat_f16, const void *vhat_f16, int B,
                             int N, int H, int Hkv, int dh, int vis_begin, int Nv, void *o_f16,
                             bool want_cues, void *ws, const float **partial_out, hipStream_t st)
{
    if (!q_f16 || !khat_f16 || !vhat_f16 || !o_f16 || !ws) return QUOTA_ERR_NULL;
    if (B <= 0 || N < 0 || H <= 0 || Hkv <= 0 || vis_begin < 0 || Nv < 0 || vis_begin + Nv > N)
        return QUOTA_ERR_INVALID_ARG;
    if ((dh != 64 && dh != 128) || H % Hkv != 0) return QUOTA_ERR_SHAPE;
    if (partial_out) *partial_out = nullptr;
    if (N == 0) return QUOTA_OK;
    float *lse2 = (float *)ws;
    float *partial = lse2 + (size_t)B * H * N;
    float scale_log2 = 1.4426950408889634f / sqrtf((float)dh);
    dim3 g1((N + 127) / 128, H, B), blk(256);
    const f16 *q = (const f16 *)q_f16, *k = (const f16 *)khat_f16, *v = (const f16 *)vhat_f16;
    const double dM = (double)B * N, dd = (double)H * dh;
    {
        ProfScope prof(QUOTA_K_ATTENTION_FWD, 4.0 * B * dd * ((double)N * (N + 1) / 2),
                       4.0 * dM * dd + 4.0 * dM * Hkv * dh, st);
        if (dh == 128)
            attn_fwd_kernel<128><<<g1, blk, 0, st>>>(q, k, v, N, H, Hkv, (f16 *)o_f16, lse2, scale_log2);
        else
            attn_fwd_kernel<64><<<g1, blk, 0, st>>>(q, k, v, N, H, Hkv, (f16 *)o_f16, lse2, scale_log2);
    }
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    if (Nv > 0 && want_cues) {
        dim3 g2((Nv + 127) / 128, H, B);
        // (query, visual key) pairs under the causal mask
        const double pairs = (double)Nv * (N - vis_begin) - (double)Nv * (Nv - 1) / 2;
        ProfScope prof(QUOTA_K_ATTENTION_COLMASS, 2.0 * B * dd * pairs, 2.0 * dM * dd + 2.0 * dM * Hkv * dh, st);
        if (dh == 128)
            colmass_kernel<128><<<g2, blk, 0, st>>>(q, k, lse2, N, H, Hkv, vis_begin, Nv, partial, scale_log2);
        else
            colmass_kernel<64><<<g2, blk, 0, st>>>(q, k, lse2, N, H, Hkv, vis_begin, Nv, partial, scale_log2);
        QUOTA_RETURN_IF_LAUNCH_FAILED();
        if (partial_out) *partial_out = partial;
    }
    return QUOTA_OK;
}

extern "C" int quota_attention_prefill_gqa(const void *q_f16, const void *khat_f16,
                                           const void *vhat_f16, int B, int N, int H, int Hkv, int dh,
                                           int vis_begin, int Nv, void *o_f16, float *cm_inter,
                                           float *cm_intra, void *ws, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const float *partial = nullptr;
    int rc = quota_internal_attention(q_f16, khat_f16, vhat_f16, B, N, H, Hkv, dh, vis_begin, Nv, o_f16,
                                      cm_inter || cm_intra, ws, &partial, st);
    if (rc != QUOTA_OK) return rc;
    if (partial) {
        colmass_reduce_kernel<<<dim3((B * Nv + 255) / 256), dim3(256), 0, st>>>(partial, B, H, Nv,
                                                                                cm_inter, cm_intra);
        QUOTA_RETURN_IF_LAUNCH_FAILED();
    }
    return QUOTA_OK;
}

// ---- the same call for callers that cannot allocate ---------------------------------------
// The row log-sum-exp and the per-head column masses (the two intermediates the call above keeps
// in the caller's workspace) live in a file-scope device array instead.  Host code never uses the
// array's name as an address: each device's copy is looked up once with hipGetSymbolAddress, with
// that device current, and the kernels receive the looked-up pointer like any other buffer.
// Every element the cue pass and the head mean read has been written earlier in the same call,
// so nothing needs clearing between calls.
static __device__ __align__(256) float attn_scratch[3 * QUOTA_ATTENTION_STATIC_MAX_ROWS];

namespace {
constexpr int kMaxDevices = 64;
float *attn_scratch_ptr[kMaxDevices];      // per device, null until the first call on it
}

extern "C" int quota_attention_prefill_static(const void *q_f16, const void *khat_f16,
                                              const void *vhat_f16, int B, int N, int H, int Hkv,
                                              int dh, int vis_begin, int Nv, void *o_f16,
                                              float *cm_inter, float *cm_intra, void *stream)
{
    if (B <= 0 || N < 0 || H <= 0) return QUOTA_ERR_INVALID_ARG;
    if ((long)B * H * N > (long)QUOTA_ATTENTION_STATIC_MAX_ROWS) return QUOTA_ERR_CAPACITY;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return QUOTA_ERR_HIP;
    if (!attn_scratch_ptr[dev]) {
        float *p = nullptr;
        if (hipGetSymbolAddress((void **)&p, HIP_SYMBOL(attn_scratch)) != hipSuccess || !p)
            return QUOTA_ERR_HIP;
        attn_scratch_ptr[dev] = p;
    }
    return quota_attention_prefill_gqa(q_f16, khat_f16, vhat_f16, B, N, H, Hkv, dh, vis_begin, Nv,
                                       o_f16, cm_inter, cm_intra, attn_scratch_ptr[dev], stream);
}

extern "C" int quota_attention_prefill(const void *q_f16, const void *khat_f16,
                                       const void *vhat_f16, int B, int N, int H, int dh,
                                       int vis_begin, int Nv, void *o_f16, float *cm_inter,
                                       float *cm_intra, void *ws, void *stream)
{
    return quota_attention_prefill_gqa(q_f16, khat_f16, vhat_f16, B, N, H, H, dh, vis_begin, Nv, o_f16,
                                       cm_inter, cm_intra, ws, stream);
}
