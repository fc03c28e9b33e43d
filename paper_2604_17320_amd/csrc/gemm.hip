// W4A4 GEMM for gfx950: int4 codes are unpacked to int8 and contracted with
// v_mfma_i32_32x32x32_i8; the per-group weight scales are applied in fp32
// inside the K loop (one convert + one fma per output element and group).
//
// Unpack trick: a nibble placed in the HIGH half of a byte is the int8 value
// 16*code (two's complement carries the sign), so "(w << 4) & 0xF0F0F0F0" and
// "w & 0xF0F0F0F0" turn one packed dword into two dwords of int8 without any
// sign-extension arithmetic.  Both operands are shifted, every group
// accumulator is therefore exactly 256x the true integer dot product; the
// factor 2^-8 is folded into the token scale (exact in fp32).
//
// Data flow per 128-deep group:
//   activations: global (packed) -> registers -> unpack -> LDS (int8, shared by
//                the 4 waves) -> MFMA A fragments
//   weights:     global (packed) -> registers -> unpack -> MFMA B fragments.
//                The 4 waves of a workgroup own disjoint column ranges, so a
//                weight is needed by exactly one wave and never touches LDS.
// The order of k inside a group does not matter for an integer dot product,
// so both operands just use the same assignment of elements to MFMA k-slots:
// a 16-byte packed chunk c (32 codes) yields "even" (low nibbles) and "odd"
// (high nibbles) int8 vectors; lane half h of k-step ks takes the even (ks
// even) or odd (ks odd) vector of chunk 2*h + ks/2.
#include "common.h"
#include "internal.h"
#include "ropequant.h"
#include "gemm_common.h"

namespace {

constexpr int AROW = 9;     // LDS row stride in 16-byte units: 8 data + 1 pad (conflict-free b128)

// Workgroup tile (32*TM) x (128*TN); wave w owns columns [w*32*TN, (w+1)*32*TN).
// CH > 0: the LDS stage holds CH groups of activations, so the workgroup meets at a
// barrier once per CH groups instead of once per group (DEPTH must be a multiple of CH).
template <int TM, int TN, int DEPTH, int CH, bool PIPE, bool ACC_OUT, bool QKV, int WPE>
__global__ __launch_bounds__(256, WPE) void w4a4_gemm_kernel(
    const uint8_t *__restrict__ qa, const float *__restrict__ sa, int M, int K, int G,
    const uint4 *__restrict__ wp, const f16 *__restrict__ sw, int N, f16 *__restrict__ y, int ldy,
    const f16 *__restrict__ res, int ldr, int32_t *__restrict__ acc_out, int tiles_m, int tiles_n,
    int vec_store, quota_qkv_epilogue qe)
{
    constexpr int BM = 32 * TM, WN = 32 * TN, BN = 4 * WN;
    constexpr int LA = (BM * 4 + 255) / 256;         // 16-byte activation loads per thread per group
    constexpr int CROW = WN + 8;                     // halves per staged output row (16-byte pad)
    constexpr int ASTAGE = BM * AROW + 2;            // uint4 per group of activations in LDS (+ spare slot)
    constexpr bool CHUNK = CH > 0;
    constexpr int CHN = CHUNK ? CH : 1;
    static_assert(DEPTH % CHN == 0, "DEPTH must be a multiple of CH");
    constexpr int TROW = BN + 8;                     // halves per row of the workgroup-wide QKV tile
    constexpr int LDS_A = 2 * CHN * ASTAGE, LDS_C = (QKV ? 32 * TROW : 4 * 32 * CROW) / 8;     // in uint4
    __shared__ uint4 lds_raw[LDS_A > LDS_C ? LDS_A : LDS_C];

    const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hl = lane >> 5;
    const int Kb = K >> 1;   // bytes per packed activation row

    // Global loads are unconditional with clamped addresses (no branches in the
    // main loop): rows past M or N repeat the last row and are never stored; a
    // chunk past the end of a ragged K repeats the last chunk and meets the
    // zero padding of the packed weights.  Addresses are a wave-uniform base
    // that advances with the group plus a loop-invariant 32-bit lane offset.
    unsigned oa[LA];                // byte offset of this thread's activation chunk in group 0
    int ca[LA], la[LA];
    bool a_on[LA];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        int i = tid + 256 * j, row = i >> 2, c = i & 3;
        a_on[j] = row < BM;
        row = min(row, BM - 1);
        ca[j] = c * 16;
        oa[j] = (unsigned)(min(m0 + row, M - 1) - m0) * (unsigned)Kb;
        la[j] = a_on[j] ? row * AROW + 2 * c : BM * AROW;   // spare slot after the tile
    }
    const uint8_t *abase = qa + (size_t)m0 * Kb;
    unsigned ow[TN], os[TN];        // uint4 / f16 index of this lane's weight chunk / scale in group 0
    int ncol[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        ncol[j] = n0 + wave * WN + 32 * j + l32;
        int n = min(ncol[j], N - 1);
        ow[j] = (unsigned)n * 4 + 2 * hl;
        os[j] = (unsigned)n;
    }

    uint4 ra[CHUNK ? CHN : DEPTH][LA], rw[DEPTH][TN][2];
    f16 rs[DEPTH][TN];
    auto load_w = [&](int stage, int g) {
        g = min(g, G - 1);
        const uint4 *wg = wp + (size_t)g * N * 4;        // uniform
        const f16 *sg = sw + (size_t)g * N;              // uniform
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            rw[stage][j][0] = wg[ow[j]];
            rw[stage][j][1] = wg[ow[j] + 1];
            rs[stage][j] = sg[os[j]];
        }
    };
    auto load_a = [&](int stage, int g) {
        g = min(g, G - 1);
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            int kb = min(g * 64 + ca[j], Kb - 16);
            ra[stage][j] = *reinterpret_cast<const uint4 *>(abase + oa[j] + (unsigned)kb);
        }
    };
    auto store_a = [&](int stage, uint4 *dst) {
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            uint4 lo, hi;
            unpack16(ra[stage][j], lo, hi);
            dst[la[j]] = lo;            // threads without a row write the spare slot
            dst[la[j] + 1] = hi;
        }
    };

    constexpr int T = TM * TN;
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
    const int fra = l32 * AROW + 4 * hl;       // this lane's A fragment (row l32 of a 32-row block)

#pragma unroll
    for (int s = 0; s < DEPTH; ++s) load_w(s, s);
    if (CHUNK) {
#pragma unroll
        for (int s = 0; s < CHN; ++s) load_a(s, s);
#pragma unroll
        for (int s = 0; s < CHN; ++s) store_a(s, lds_raw + s * ASTAGE);
    } else {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) load_a(s, s);
        store_a(0, lds_raw);
    }
    __syncthreads();
    int cb = 0;                     // CHUNK: which half of the LDS buffer holds the current groups

    // Software pipeline over the 32x32 sub-tiles, carried across groups: while the
    // matrix core runs the 4 MFMAs of a sub-tile, the vector ALU applies the group
    // scale (one convert + one fma per element) to the previous sub-tile -- for the
    // first sub-tile of a group that is the last sub-tile of the group before.
    i32x16 pend = i32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};   // sub-tile awaiting its scale
    float sw_prev = 0.0f;           // scale that goes with the pending sub-tile
    bool live_prev = false;
    auto scale_in = [&](int t, const i32x16 &a, float scale, bool live) {
        const int i = t / TN, j = t % TN;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            yacc[i][j][r] = __builtin_fmaf((float)a[r], scale, yacc[i][j][r]);
            if (ACC_OUT) tot[i][j][r] += live ? a[r] : 0;
        }
    };

    auto unpack_w = [&](int stage, int g, i32x4 (&fb)[TN][4], float (&swn)[TN]) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            swn[j] = (g < G && ncol[j] < N) ? (float)rs[stage][j] : 0.0f;
            uint4 lo, hi;
            unpack16(rw[stage][j][0], lo, hi);
            fb[j][0] = as_i32x4(lo);
            fb[j][1] = as_i32x4(hi);
            unpack16(rw[stage][j][1], lo, hi);
            fb[j][2] = as_i32x4(lo);
            fb[j][3] = as_i32x4(hi);
        }
    };
    auto read_a = [&](const uint4 *abuf, i32x4 (&fa)[TM][4]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) fa[i][ks] = as_i32x4(abuf[fra + 32 * i * AROW + ks]);
    };
    // MFMAs of group g with the scale of the previous sub-tile interleaved
    auto mfma_group = [&](const i32x4 (&fa)[TM][4], const i32x4 (&fb)[TN][4], const float (&swn)[TN], int g) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int i = t / TN, j = t % TN;
            i32x16 a = i32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                a = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i][ks], fb[j][ks], a, 0, 0, 0);
            if (t == 0) scale_in(T - 1, pend, sw_prev, live_prev);
            else scale_in(t - 1, pend, swn[(t - 1) % TN], g < G);
            pend = a;
        }
        sw_prev = swn[(T - 1) % TN];
        live_prev = g < G;
    };

    const int Gpad = (G + DEPTH - 1) / DEPTH * DEPTH;
    if constexpr (PIPE) {
        // Group-level software pipeline for the narrow tiles, where little else hides
        // latency: while the MFMAs of group g run, the weights of group g+1 are unpacked and
        // its activation fragments are already on their way from LDS.  Scheduling barriers
        // pin the phases of an iteration; without them the fragment reads sink next to their
        // first use and every MFMA waits on LDS.
        static_assert(CHUNK && DEPTH % 2 == 0, "PIPE needs chunked staging and an even DEPTH");
        i32x4 fbp[2][TN][4], fap[2][TM][4];
        float swp[2][TN];
        unpack_w(0, 0, fbp[0], swp[0]);
        read_a(lds_raw, fap[0]);
#pragma unroll 1
        for (int g0 = 0; g0 < Gpad; g0 += DEPTH) {
#pragma unroll
            for (int s = 0; s < DEPTH; ++s) {
                const int g = g0 + s, cur = s & 1, nxt = cur ^ 1, s1 = (s + 1) % DEPTH;
                const bool chunk_end = s % CHN == CHN - 1;
                if (s % CHN == 0) {             // activations of the next CH groups -> registers
#pragma unroll
                    for (int c = 0; c < CHN; ++c) load_a(c, g + CHN + c);
                }
                load_w(s, g + DEPTH);           // stage s was unpacked during the previous group
                if (!chunk_end) read_a(lds_raw + (cb * CHN + s % CHN + 1) * ASTAGE, fap[nxt]);
                __builtin_amdgcn_sched_barrier(0);
                mfma_group(fap[cur], fbp[cur], swp[cur], g);
                unpack_w(s1, g + 1, fbp[nxt], swp[nxt]);
#pragma unroll
                for (int q = 0; q < 4 * T; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, (ACC_OUT ? 12 : 8) + 6 / TM, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (chunk_end) {                // next CH groups of activations -> the other half
#pragma unroll
                    for (int c = 0; c < CHN; ++c) store_a(c, lds_raw + ((cb ^ 1) * CHN + c) * ASTAGE);
                    __syncthreads();
                    cb ^= 1;
                    read_a(lds_raw + cb * CHN * ASTAGE, fap[nxt]);
                }
            }
        }
    } else {
#pragma unroll 1
    for (int g0 = 0; g0 < Gpad; g0 += DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            const int g = g0 + s;
            if (CHUNK && s % CHN == 0) {        // activations of the next CH groups -> registers
#pragma unroll
                for (int c = 0; c < CHN; ++c) load_a(c, g + CHN + c);
            }
            const uint4 *abuf = lds_raw + (CHUNK ? (cb * CHN + s % CHN) : (g & 1)) * ASTAGE;
            // activation fragments of group g from LDS, weights of group g from registers
            i32x4 fa[TM][4], fb[TN][4];
            float swn[TN];
            read_a(abuf, fa);
            unpack_w(s, g, fb, swn);
            // the stage that held group g is free again: prefetch group g + DEPTH into it
            // (its activation registers were stored to LDS one iteration ago)
            load_w(s, g + DEPTH);
            if (!CHUNK) load_a(s, g + DEPTH);
            mfma_group(fa, fb, swn, g);
            // issue order hint: 1 MFMA : 8 VALU
#pragma unroll
            for (int q = 0; q < 4 * T; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, ACC_OUT ? 12 : 8, 0);
            }
            if (!CHUNK) {           // activations of group g+1 -> the other LDS buffer
                store_a((s + 1) % DEPTH, lds_raw + ((g & 1) ^ 1) * ASTAGE);
                __syncthreads();
            }
            if (CHUNK && s % CHN == CHN - 1) {  // activations of the next CH groups -> the other half
#pragma unroll
                for (int c = 0; c < CHN; ++c) store_a(c, lds_raw + ((cb ^ 1) * CHN + c) * ASTAGE);
                __syncthreads();
                cb ^= 1;
            }
        }
    }
    }
    scale_in(T - 1, pend, sw_prev, live_prev);

    // epilogue: token scale (with the 2^-8 of the shifted operands), residual, fp16.
    // With an aligned output the fp16 tile goes through LDS (the activation buffers
    // are free after the last barrier) so that every lane stores 16 contiguous bytes.
    if constexpr (QKV) {
        // Fused epilogue of the QKV projection: the fp16 tile (whole heads: the tile width
        // divides the model width and is a multiple of the head size) is staged in LDS by all
        // four waves; then every thread takes (row, 8-channel chunk) items and applies RoPE at
        // the token's position id (q and k tiles) and the 4-bit K/V group quantizer (k and v
        // tiles) exactly as the stand-alone kernel does.  q | k | v are column ranges
        // [0,d) [d,d+dkv) [d+dkv,d+2dkv), so a tile lies in one of them.
        f16 *tile = reinterpret_cast<f16 *>(lds_raw);
        const int d = qe.d, dkv = qe.dkv;
        const int region = n0 < d ? 0 : (n0 < d + dkv ? 1 : 2);          // tile-uniform
        const int c0 = n0 - (region == 0 ? 0 : (region == 1 ? d : d + dkv));
        const int CPH = qe.dh >> 3, HALF = CPH >> 1, cpr = dkv >> 3, gpr = dkv >> 6;
        const int row_step = qe.row_step ? min(max(*qe.row_step, 0), qe.max_steps - 1) : 0;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (i) __syncthreads();                   // the previous row block has been read
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r >> 2) + 4 * hl + (r & 3);
                const int m = m0 + 32 * i + row;
                const float sam = sa[m < M ? m : M - 1] * 0.00390625f;
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    tile[row * TROW + wave * WN + 32 * j + l32] = to_f16(yacc[i][j][r] * sam);
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < 32 * (BN / 8) / 256; ++q) {
                const int idx = q * 256 + tid, row = idx / (BN / 8), c = idx % (BN / 8);
                const int m = m0 + 32 * i + row;
                const bool m_ok = m < M;
                const int mm = m_ok ? m : M - 1;
                Pack16 x, xp, out;
                x.u = *reinterpret_cast<const uint4 *>(tile + row * TROW + 8 * c);
                if (y && m_ok) *reinterpret_cast<uint4 *>(y + (size_t)m * ldy + n0 + 8 * c) = x.u;
                const int col = c0 + 8 * c;           // first channel of the chunk inside q, k or v
                if (region < 2) {
                    const int cc = c % CPH;
                    xp.u = *reinterpret_cast<const uint4 *>(tile + row * TROW + 8 * (c ^ HALF));
                    const int pr = min(max(qe.pos[mm], 0), qe.n_pos - 1);
                    const float *cp = qe.cosT + (size_t)pr * (qe.dh >> 1) + 8 * (cc % HALF);
                    const float *sp = qe.sinT + (size_t)pr * (qe.dh >> 1) + 8 * (cc % HALF);
                    float cs[8], sn[8];
                    *reinterpret_cast<float4 *>(cs) = *reinterpret_cast<const float4 *>(cp);
                    *reinterpret_cast<float4 *>(cs + 4) = *reinterpret_cast<const float4 *>(cp + 4);
                    *reinterpret_cast<float4 *>(sn) = *reinterpret_cast<const float4 *>(sp);
                    *reinterpret_cast<float4 *>(sn + 4) = *reinterpret_cast<const float4 *>(sp + 4);
                    rope8(x, xp, cs, sn, cc >= HALF, out);
                } else {
                    out = x;
                }
                if (region == 0) {
                    if (m_ok) *reinterpret_cast<uint4 *>(qe.q_rot + (size_t)m * d + col) = out.u;
                } else {
                    float f[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[e] = (float)out.h[e];
                    Pack16 hat;
                    f16 sc;
                    const uint32_t word = kv_quant8(f, &sc, &hat);     // all 8 lanes of a group take part
                    if (m_ok) {
                        f16 *xh = region == 1 ? qe.khat : qe.vhat;
                        uint32_t *codes = region == 1 ? qe.k_codes : qe.v_codes;
                        f16 *scales = region == 1 ? qe.k_scales : qe.v_scales;
                        *reinterpret_cast<uint4 *>(xh + (size_t)m * dkv + col) = hat.u;
                        const size_t orow = (size_t)m * qe.code_row_stride + qe.code_row_offset + row_step;
                        codes[orow * cpr + (col >> 3)] = word;
                        if ((c & 7) == 0) scales[orow * gpr + (col >> 6)] = sc;
                    }
                }
            }
        }
        return;
    }
    f16 *cw = reinterpret_cast<f16 *>(lds_raw) + wave * 32 * CROW;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 8 * (r >> 2) + 4 * hl + (r & 3);
            const int m = m0 + 32 * i + row;
            const bool m_ok = m < M;
            const float sam = sa[m_ok ? m : M - 1] * 0.00390625f;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = ncol[j];
                const bool ok = m_ok && n < N;
                float v = yacc[i][j][r] * sam;
                if (res && ok) v = v + (float)res[(size_t)m * ldr + n];
                const f16 h = to_f16(v);
                if (vec_store) cw[row * CROW + 32 * j + l32] = h;
                else if (y && ok) y[(size_t)m * ldy + n] = h;
                if (ACC_OUT && ok) acc_out[(size_t)m * N + n] = tot[i][j][r] >> 8;
            }
        }
        if (vec_store) {
            __syncthreads();                      // staged tile visible (also fences the type-punned LDS accesses)
#pragma unroll
            for (int q = 0; q < 32 * (WN / 8) / 64; ++q) {
                const int idx = q * 64 + lane, row = idx / (WN / 8), ch = idx % (WN / 8);
                const int m = m0 + 32 * i + row, n = n0 + wave * WN + 8 * ch;
                const uint4 v = *reinterpret_cast<const uint4 *>(cw + row * CROW + 8 * ch);
                if (m < M && n < N) *reinterpret_cast<uint4 *>(y + (size_t)m * ldy + n) = v;
            }
            __syncthreads();
        }
    }
}

// ---- at most 16 rows (the decode step): weight streaming -------------------------------
// With M <= 16 the GEMM has too few outputs to fill the chip with one accumulation chain per
// wave, and the fp32 chain over groups cannot be split.  The exact int32 group sums can: in a round
// the 8 waves of a workgroup take U groups each (group r0 + 8 u + w for wave w: all their loads in
// flight together, U * 8 groups = 2 KB of weights per column block and round), park their 16 x 16
// int32 results in LDS, and one thread per output then runs the fp32 chain over those 8 U groups in
// ascending order.  Operands need no LDS: for v_mfma_i32_16x16x64_i8 a lane owns (row or column
// l % 16, 16 k-slots l / 16), so lane l loads the 16 packed bytes (32 codes) number l / 16 of its
// row's group for A and of its column's group for B, and the even / odd nibble vectors feed two
// MFMAs.  NB = 16-column blocks per workgroup.
template <int NB, int U>
__global__ __launch_bounds__(512) void w4a4_gemv16_kernel(
    const uint8_t *__restrict__ qa, const float *__restrict__ sa, int M, int K, int G,
    const uint4 *__restrict__ wp, const f16 *__restrict__ sw, int N, f16 *__restrict__ y, int ldy,
    const f16 *__restrict__ res, int ldr)
{
    constexpr int R = 8 * U;                    // groups per round
    __shared__ int accs[R][NB][4][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 15, q = lane >> 4;
    const int n0 = blockIdx.x * 16 * NB, Kb = K >> 1;
    const uint8_t *arow = qa + (size_t)min(c, M - 1) * Kb;

    // chain ownership: thread t < 256 * NB owns the output held by (block j, register reg, lane ol)
    const int oj = tid >> 8, oreg = (tid >> 6) & 3, ol = tid & 63;
    const bool owner = tid < 256 * NB;
    const int om = 4 * (ol >> 4) + oreg, on = n0 + 16 * oj + (ol & 15);
    float y32 = 0.0f;

    // The R x (16 NB) group scales of a round come in with ONE 8-byte load per lane of waves 0..NB-1
    // (lane l: group l / 4 of the round, 4 columns) and reach the chain owners through LDS, transposed
    // so that an owner reads its column's R scales as two 16-byte pieces: a vector-memory instruction
    // costs a wave tens of issue cycles, and R of them per owner and round were a third of the round.
    static_assert(R == 16, "the scale staging below is laid out for 16 groups per round");
    __shared__ __align__(16) f16 scs[16 * NB][R];
    uint4 ra[U], rb[U][NB];
    uint2 rsv = make_uint2(0, 0);
    auto fetch = [&](int r0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = min(r0 + 8 * u + wave, G - 1);
            ra[u] = *reinterpret_cast<const uint4 *>(arow + min(g * 64 + q * 16, Kb - 16));
#pragma unroll
            for (int j = 0; j < NB; ++j) rb[u][j] = wp[((size_t)g * N + n0 + 16 * j + c) * 4 + q];
        }
        if (wave < NB)
            rsv = *reinterpret_cast<const uint2 *>(sw + (size_t)min(r0 + (lane >> 2), G - 1) * N + n0 + 16 * wave +
                                                   4 * (lane & 3));
    };
    fetch(0);
    for (int r0 = 0; r0 < G; r0 += R) {
        i32x4 acc[U][NB];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint4 alo, ahi;
            unpack16(ra[u], alo, ahi);
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                uint4 blo, bhi;
                unpack16(rb[u][j], blo, bhi);
                acc[u][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_i32x4(alo), as_i32x4(blo), i32x4{0, 0, 0, 0}, 0, 0, 0);
                acc[u][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_i32x4(ahi), as_i32x4(bhi), acc[u][j], 0, 0, 0);
            }
        }
        if (wave < NB) {                            // this round's scales -> LDS, [column][group]
            const int col = 16 * wave + 4 * (lane & 3), gi = lane >> 2;
            Pack16 t;
            t.u = make_uint4(rsv.x, rsv.y, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) scs[col + e][gi] = t.h[e];
        }
        bool live[U];
#pragma unroll
        for (int u = 0; u < U; ++u) live[u] = r0 + 8 * u + wave < G;
        if (r0 + R < G) fetch(r0 + R);              // next round's loads fly during the exchange
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) accs[8 * u + wave][j][i][lane] = live[u] ? acc[u][j][i] : 0;
        __syncthreads();
        if (owner) {
            Pack16 s0, s1;
            const uint4 *sp = reinterpret_cast<const uint4 *>(&scs[16 * oj + (ol & 15)][0]);
            s0.u = sp[0];
            s1.u = sp[1];
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const float sc = r0 + i < G ? (float)(i < 8 ? s0.h[i] : s1.h[i - 8]) : 0.0f;
                y32 = __builtin_fmaf((float)accs[i][oj][oreg][ol], sc, y32);
            }
        }
        __syncthreads();
    }
    if (owner && om < M) {
        float v = y32 * (sa[om] * 0.00390625f);
        if (res) v = v + (float)res[(size_t)om * ldr + on];
        y[(size_t)om * ldy + on] = to_f16(v);
    }
}

template <int NB, int U>
int launch_gemv16(const uint8_t *qa, const float *sa, int M, const quota_weights *W, f16 *y, int ldy,
                  const f16 *res, int ldr, hipStream_t st)
{
    const int G = (W->K + QUOTA_GROUP_W - 1) / QUOTA_GROUP_W;
    const double Md = M, Nd = W->N, Kd = W->K;
    ProfScope prof(QUOTA_K_GEMM_ROWS16, 2.0 * Md * Nd * Kd,
                   Nd * Kd / 2 + 2.0 * Nd * G + Md * Kd / 2 + 4 * Md + 2.0 * Md * Nd * (res ? 2 : 1), st);
    w4a4_gemv16_kernel<NB, U><<<dim3(W->N / (16 * NB)), dim3(512), 0, st>>>(
        qa, sa, M, W->K, G, (const uint4 *)W->packed, (const f16 *)W->scales, W->N, y, ldy, res, ldr);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

template <int TM, int TN, int DEPTH, int CH, bool PIPE, bool ACC_OUT, bool QKV = false, int WPE = 1>
int launch(int kernel_id, const uint8_t *qa, const float *sa, int M, const quota_weights *W, f16 *y,
           int ldy, const f16 *res, int ldr, int32_t *acc, hipStream_t st,
           const quota_qkv_epilogue *qe = nullptr)
{
    constexpr int BM = 32 * TM, BN = 128 * TN;
    int G = (W->K + QUOTA_GROUP_W - 1) / QUOTA_GROUP_W;
    int tiles_m = (M + BM - 1) / BM, tiles_n = (W->N + BN - 1) / BN;
    const double Md = M, Nd = W->N, Kd = W->K;
    ProfScope prof(kernel_id, 2.0 * Md * Nd * Kd,
                   Nd * Kd / 2 + 2.0 * Nd * G + Md * Kd / 2 + 4 * Md +
                       (QKV ? Md * (Nd / 3) * (7 + 1.0 / 16) + 4 * Md : 2.0 * Md * Nd * (res ? 2 : 1)), st);
    static const quota_qkv_epilogue no_qe = {};
    w4a4_gemm_kernel<TM, TN, DEPTH, CH, PIPE, ACC_OUT, QKV, WPE><<<dim3(tiles_m * tiles_n), dim3(256), 0, st>>>(
        qa, sa, M, W->K, G, (const uint4 *)W->packed, (const f16 *)W->scales, W->N, y, ldy, res, ldr,
        acc, tiles_m, tiles_n, (y && ldy % 8 == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0) ? 1 : 0,
        qe ? *qe : no_qe);
    QUOTA_RETURN_IF_LAUNCH_FAILED();
    return QUOTA_OK;
}

}  // namespace

// Tile choice by a small cost model fitted to measured kernel times on this GPU (us).
// W workgroups run R at a time per CU on 256 CUs; a launch that fits (W <= 256 R) costs
// c0 + G * u[workgroups per CU - 1], a larger one c0 + G * u[R-1] * (f0 + f1 * W / (256 R)).
// Wide tiles reuse each unpacked weight for 64 rows but need full rounds; the 32-row tiles
// spread small problems over more waves; the deep variant prefetches weights 8 groups
// ahead for launches of at most one workgroup per CU; the lean 64x128 variant (no group
// pipeline, registers capped so that three workgroups fit on a CU) takes the launches that
// would need a second round of the pipelined one.  `allow_wide` = false leaves the
// 256-column tile out.
static int g_gemm_variant = -1;      // -1: chosen per launch; else pinned by quota_set_gemm_variant

extern "C" int quota_set_gemm_variant(int variant)
{
    if (variant < -1 || variant > 4) return QUOTA_ERR_INVALID_ARG;
    g_gemm_variant = variant;
    return QUOTA_OK;
}

static int choose_tile(int M, int N, int K, bool allow_wide)
{
    struct Tile { int bm, bn, R; float c0, u[3], f0, f1; };
    static const Tile tiles[5] = {
        {64, 256, 2, 13.0f, {0.69f, 1.34f, 0.0f}, 0.0f, 1.22f},     // <2,2,3,0>
        {64, 128, 2, 6.0f, {0.39f, 0.69f, 0.0f}, 0.0f, 1.27f},      // <2,1,4,2> pipelined
        {32, 128, 3, 0.5f, {0.39f, 0.61f, 0.82f}, 0.35f, 0.92f},    // <1,1,4,2> pipelined
        {32, 128, 2, 4.0f, {0.27f, 0.46f, 0.0f}, 0.0f, 1.45f},      // <1,1,8,4> pipelined, deep prefetch
        {64, 128, 3, 6.0f, {0.53f, 0.75f, 1.06f}, 0.0f, 1.3f},      // <2,1,3,0>, three workgroups per CU
    };
    if (g_gemm_variant >= (allow_wide ? 0 : 1) && g_gemm_variant < 5) return g_gemm_variant;
    const int G = (K + QUOTA_GROUP_W - 1) / QUOTA_GROUP_W;
    int best = -1;
    float best_t = 0.0f;
    for (int i = allow_wide ? 0 : 1; i < 5; ++i) {
        const Tile &t = tiles[i];
        const long wgs = (long)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
        const float x = (float)wgs / (256.0f * t.R);
        // a launch that spills into a second round pays for most of that round (measured: >= 1.6x)
        const float over = t.f0 + t.f1 * x;
        const float est = x <= 1.0f ? t.c0 + G * t.u[(wgs + 255) / 256 - 1]
                                    : t.c0 + G * t.u[t.R - 1] * (i == 1 && over < 1.6f ? 1.6f : over);
        if (best < 0 || est < best_t) { best = i; best_t = est; }
    }
    return best;
}

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
    if (acc_i32_opt)
        return launch<2, 1, 2, 0, false, true>(QUOTA_K_GEMM_OTHER, qa, sa, M, W, y, ldy, res, ldr, acc_i32_opt, st);
    if (M <= 16)            // the decode step: stream the weights once, groups spread over 8 waves
        return W->N <= 8192 ? launch_gemv16<1, 2>(qa, sa, M, W, y, ldy, res, ldr, st)
                            : launch_gemv16<2, 2>(qa, sa, M, W, y, ldy, res, ldr, st);
    switch (choose_tile(M, W->N, W->K, true)) {
    case 0: return launch<2, 2, 3, 0, false, false>(QUOTA_K_GEMM_64X256, qa, sa, M, W, y, ldy, res, ldr, nullptr, st);
    case 1: return launch<2, 1, 4, 2, true, false>(QUOTA_K_GEMM_64X128, qa, sa, M, W, y, ldy, res, ldr, nullptr, st);
    case 2: return launch<1, 1, 4, 2, true, false>(QUOTA_K_GEMM_32X128, qa, sa, M, W, y, ldy, res, ldr, nullptr, st);
    case 3: return launch<1, 1, 8, 4, true, false>(QUOTA_K_GEMM_32X128_DEEP, qa, sa, M, W, y, ldy, res, ldr, nullptr, st);
    default: return launch<2, 1, 3, 0, false, false, false, 3>(QUOTA_K_GEMM_64X128_LEAN, qa, sa, M, W, y, ldy, res, ldr, nullptr, st);
    }
}

// QKV projection with the RoPE + 4-bit K/V quantizer fused into the epilogue (see the kernel).
// y_opt, when not null, also receives the plain fp16 q | k | v.  Returns QUOTA_ERR_SHAPE when the
// shape does not fit the fused form (the caller then runs the two kernels separately).
int quota_internal_w4a4_gemm_qkv(const uint8_t *qa, const float *sa, int M, const quota_weights *W,
                                 void *y_opt, const quota_qkv_epilogue *qe, hipStream_t st)
{
    if (!qa || !sa || !W || !W->packed || !W->scales || !qe || !qe->pos || !qe->cosT || !qe->sinT ||
        !qe->q_rot || !qe->khat || !qe->vhat || !qe->k_codes || !qe->k_scales || !qe->v_codes || !qe->v_scales)
        return QUOTA_ERR_NULL;
    if (M < 0 || qe->n_pos <= 0) return QUOTA_ERR_INVALID_ARG;
    const int d = qe->d, dkv = qe->dkv;
    if ((qe->dh != 64 && qe->dh != 128) || d <= 0 || d % 128 != 0 || dkv <= 0 || dkv % 128 != 0 ||
        W->N != d + 2 * dkv || W->K % 32 != 0)
        return QUOTA_ERR_SHAPE;
    if (M == 0) return QUOTA_OK;
    f16 *y = (f16 *)y_opt;
    // (the 256-column tile is left out: with this epilogue it runs at its register limit)
    switch (choose_tile(M, W->N, W->K, false)) {
    case 1: return launch<2, 1, 4, 2, true, false, true>(QUOTA_K_GEMM_64X128, qa, sa, M, W, y, W->N, nullptr, 0, nullptr, st, qe);
    case 2: return launch<1, 1, 4, 2, true, false, true>(QUOTA_K_GEMM_32X128, qa, sa, M, W, y, W->N, nullptr, 0, nullptr, st, qe);
    case 3: return launch<1, 1, 8, 4, true, false, true>(QUOTA_K_GEMM_32X128_DEEP, qa, sa, M, W, y, W->N, nullptr, 0, nullptr, st, qe);
    default: return launch<2, 1, 3, 0, false, false, true, 3>(QUOTA_K_GEMM_64X128_LEAN, qa, sa, M, W, y, W->N, nullptr, 0, nullptr, st, qe);
    }
}
