// Row-quantizer pieces shared by the row kernels.  A row is owned by a GROUP of threads (one wave,
// or a whole 256-thread workgroup) and cached in registers as 16-byte chunks: chunk c belongs to
// thread c % GROUP of the group, as its (c / GROUP)-th chunk.
#pragma once
#include "common.h"

#define ROW_THREADS 256
#define ROW_MAXCHUNK 16  // workgroup-per-row kernels: 16 chunks * 8 halves * 256 threads = 32768 columns
#define ROW_MAXCOLS 32768

// final phase shared by the row kernels: quantize the cached row `v` with absmax `a`, store the
// packed codes, return this thread's share of the residual sum of squares.
template <bool WANT_RES, int GROUP, int NCH>
__device__ __forceinline__ double quantize_cached_row(const Pack16 *v, int nchunk, int idx, float a,
                                                      uint32_t *__restrict__ qrow, float &s_out)
{
    float s = 1.0f, inv = 0.0f;
    if (a != 0.0f) { s = a / 7.0f; inv = 7.0f / a; }
    s_out = s;
    double rs = 0.0;
#pragma unroll
    for (int r = 0; r < NCH; ++r) {
        int c = idx + GROUP * r;
        if (c < nchunk) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f = (float)v[r].h[e];
                const uint32_t cb = code_bits(f * inv);
                word |= (cb & 0xFu) << (4 * e);
                if (WANT_RES) {
                    float deq = code_float(cb) * s;
                    float rr = deq - f;
                    rs = __builtin_fma((double)rr, (double)rr, rs);     // product exact in fp64
                }
            }
            if (qrow) qrow[c] = word;
        }
    }
    return rs;
}
