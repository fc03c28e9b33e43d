// W4A4 GEMM for gfx950: int4 codes (activations and weights) are unpacked to
// int8 on the way into LDS and contracted with v_mfma_i32_32x32x32_i8; the
// per-group weight scales are applied in fp32 inside the K loop.
//
// Unpack trick: a nibble placed in the HIGH half of a byte is the int8 value
// 16*code (two's complement carries the sign), so "(w << 4) & 0xF0F0F0F0" and
// "w & 0xF0F0F0F0" turn one packed dword into two dwords of int8 without any
// sign-extension arithmetic.  Both operands are shifted, every group
// accumulator is therefore exactly 256x the true integer dot product; the
// factor 2^-8 is folded into the token scale (exact in fp32).
//
// The order of k inside a 128-wide group does not matter for an integer dot
// product, so both operands simply use the same unpack and the same LDS chunk
// order: chunk 2c holds the even elements of packed 16-byte chunk c, chunk
// 2c+1 the odd ones.
#include "common.h"

namespace {

template <int BM, int BN>
struct GemmSmem {
    // [stage][row][128 bytes], 16-byte chunks XOR-swizzled by (row & 7)
    uint4 a[2][BM * 8];
    uint4 b[2][BN * 8];
};

__device__ __forceinline__ void unpack16(const uint4 &v, uint4 &lo, uint4 &hi)
{
    lo.x = (v.x << 4) & 0xF0F0F0F0u; hi.x = v.x & 0xF0F0F0F0u;
    lo.y = (v.y << 4) & 0xF0F0F0F0u; hi.y = v.y & 0xF0F0F0F0u;
    lo.z = (v.z << 4) & 0xF0F0F0F0u; hi.z = v.z & 0xF0F0F0F0u;
    lo.w = (v.w << 4) & 0xF0F0F0F0u; hi.w = v.w & 0xF0F0F0F0u;
}

// XCD-aware tile id: consecutive dispatch ids go round-robin over the 8 XCDs
// (each with its own L2), so give each XCD a contiguous range of tiles.
__device__ __forceinline__ int xcd_remap(int pid, int total)
{
    int x = pid & 7, idx = pid >> 3;
    int per = total >> 3, rem = total & 7;
    return x * per + (x < rem ? x : rem) + idx;
}

template <int BM, int BN, bool ACC_OUT>
__global__ __launch_bounds__(256) void w4a4_gemm_kernel(
    const uint8_t *__restrict__ qa, const float *__restrict__ sa, int M, int K, int G,
    const uint4 *__restrict__ wp, const f16 *__restrict__ sw, int N, f16 *__restrict__ y, int ldy,
    const f16 *__restrict__ res, int ldr, int32_t *__restrict__ acc_out, int tiles_m, int tiles_n)
{
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int LA = BM * 4 / 256, LB = BN * 4 / 256;   // 16-byte loads per thread per group
    static_assert(LA >= 1 && LB >= 1, "tile too small for 256 threads");
    extern __shared__ uint4 smem_raw[];
    GemmSmem<BM, BN> &sm = *reinterpret_cast<GemmSmem<BM, BN> *>(smem_raw);

    const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, hl = lane >> 5;
    const int Kb = K >> 1;   // bytes per activation row

    uint4 ra[LA], rb[LB];
    auto load_group = [&](int g) {
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            int i = tid + 256 * j, row = i >> 2, c = i & 3;
            int m = m0 + row, kb = g * 64 + c * 16;
            ra[j] = (m < M && kb < Kb)
                        ? *reinterpret_cast<const uint4 *>(qa + (size_t)m * Kb + kb)
                        : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            int i = tid + 256 * j, row = i >> 2, c = i & 3;
            int n = n0 + row;
            rb[j] = n < N ? wp[((size_t)g * N + n) * 4 + c] : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_group = [&](int st) {
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            int i = tid + 256 * j, row = i >> 2, c = i & 3;
            uint4 lo, hi;
            unpack16(ra[j], lo, hi);
            sm.a[st][row * 8 + ((2 * c) ^ (row & 7))] = lo;
            sm.a[st][row * 8 + ((2 * c + 1) ^ (row & 7))] = hi;
        }
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            int i = tid + 256 * j, row = i >> 2, c = i & 3;
            uint4 lo, hi;
            unpack16(rb[j], lo, hi);
            sm.b[st][row * 8 + ((2 * c) ^ (row & 7))] = lo;
            sm.b[st][row * 8 + ((2 * c + 1) ^ (row & 7))] = hi;
        }
    };

    float yacc[TM][TN][16];
    int tot[ACC_OUT ? TM : 1][ACC_OUT ? TN : 1][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                yacc[i][j][r] = 0.0f;
                if (ACC_OUT) tot[i][j][r] = 0;
            }

    // this lane's output column in each 32-wide column block, and its scale
    int ncol[TN];
    float swn[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) ncol[j] = n0 + wn * WN + 32 * j + l32;
    auto load_scales = [&](int g) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
            swn[j] = ncol[j] < N ? (float)sw[(size_t)g * N + ncol[j]] : 0.0f;
    };

    load_group(0);
    store_group(0);
    __syncthreads();

    for (int g = 0; g < G; ++g) {
        const int st = g & 1;
        if (g + 1 < G) load_group(g + 1);
        load_scales(g);

        i32x4 fa[TM][4], fb[TN][4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            int ch = 2 * ks + hl;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int row = wm * WM + 32 * i + l32;
                uint4 t = sm.a[st][row * 8 + (ch ^ (row & 7))];
                fa[i][ks] = i32x4{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int row = wn * WN + 32 * j + l32;
                uint4 t = sm.b[st][row * 8 + (ch ^ (row & 7))];
                fb[j][ks] = i32x4{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                i32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i][ks], fb[j][ks], acc, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    yacc[i][j][r] = __builtin_fmaf((float)acc[r], swn[j], yacc[i][j][r]);
                    if (ACC_OUT) tot[i][j][r] += acc[r];
                }
            }
        if (g + 1 < G) store_group(st ^ 1);
        __syncthreads();
    }

    // epilogue: token scale (with the 2^-8 of the shifted operands), residual, fp16
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int m = m0 + wm * WM + 32 * i + 8 * (r >> 2) + 4 * hl + (r & 3);
            if (m >= M) continue;
            float sam = sa[m] * 0.00390625f;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = ncol[j];
                if (n >= N) continue;
                float v = yacc[i][j][r] * sam;
                if (res) v = v + (float)res[(size_t)m * ldr + n];
                if (y) y[(size_t)m * ldy + n] = to_f16(v);
                if (ACC_OUT) acc_out[(size_t)m * N + n] = tot[i][j][r] >> 8;
            }
        }
}

template <int BM, int BN, bool ACC_OUT>
int launch(const uint8_t *qa, const float *sa, int M, const quota_weights *W, f16 *y, int ldy,
           const f16 *res, int ldr, int32_t *acc, hipStream_t st)
{
    int G = (W->K + QUOTA_GROUP_W - 1) / QUOTA_GROUP_W;
    int tiles_m = (M + BM - 1) / BM, tiles_n = (W->N + BN - 1) / BN;
    size_t smem = sizeof(GemmSmem<BM, BN>);
    auto kern = w4a4_gemm_kernel<BM, BN, ACC_OUT>;
    static bool attr_set = false;      // once per tile shape; not a stream operation
    if (smem > 48 * 1024 && !attr_set) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return QUOTA_ERR_HIP;
        attr_set = true;
    }
    const double Md = M, Nd = W->N, Kd = W->K;
    ProfScope prof(BM == 128 && BN == 128 ? QUOTA_K_GEMM_128X128
                   : (BM == 64 && BN == 64 ? QUOTA_K_GEMM_64X64 : QUOTA_K_GEMM_OTHER),
                   2.0 * Md * Nd * Kd,
                   Nd * Kd / 2 + 2.0 * Nd * G + Md * Kd / 2 + 4 * Md + 2.0 * Md * Nd * (res ? 2 : 1), st);
    kern<<<dim3(tiles_m * tiles_n), dim3(256), smem, st>>>(
        qa, sa, M, W->K, G, (const uint4 *)W->packed, (const f16 *)W->scales, W->N, y, ldy, res,
        ldr, acc, tiles_m, tiles_n);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

}  // namespace

extern "C" int quota_w4a4_gemm(const uint8_t *qa, const float *sa, int M, const quota_weights *W,
                               void *y_f16, int ldy, const void *residual_opt, int ldr,
                               int32_t *acc_i32_opt, void *stream)
{
    if (!qa || !sa || !W || !W->packed || !W->scales) return QUOTA_ERR_NULL;
    if (!y_f16 && !acc_i32_opt) return QUOTA_ERR_NULL;
    if (M < 0 || W->N <= 0 || W->K <= 0) return QUOTA_ERR_INVALID_ARG;
    if (W->N % 64 != 0 || W->K % 32 != 0) return QUOTA_ERR_SHAPE;
    if (y_f16 && ldy < W->N) return QUOTA_ERR_INVALID_ARG;
    if (residual_opt && ldr < W->N) return QUOTA_ERR_INVALID_ARG;
    if (M == 0) return QUOTA_OK;
    hipStream_t st = (hipStream_t)stream;
    f16 *y = (f16 *)y_f16;
    const f16 *res = (const f16 *)residual_opt;
    if (acc_i32_opt) return launch<64, 64, true>(qa, sa, M, W, y, ldy, res, ldr, acc_i32_opt, st);
    long tiles_big = (long)((M + 127) / 128) * ((W->N + 127) / 128);
    if (tiles_big >= 256)
        return launch<128, 128, false>(qa, sa, M, W, y, ldy, res, ldr, nullptr, st);
    return launch<64, 64, false>(qa, sa, M, W, y, ldy, res, ldr, nullptr, st);
}
