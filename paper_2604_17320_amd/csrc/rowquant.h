// Row-quantizer pieces shared by the row kernels (one 256-thread workgroup per row, the row
// cached in registers as 16-byte chunks: chunk c of the row belongs to thread c % 256).
#pragma once
#include "common.h"

#define ROW_THREADS 256
#define ROW_MAXCHUNK 8   // 8 chunks * 8 halves * 256 threads = 16384 columns

// final phase shared by the three row kernels: quantize the cached row `v`
// with absmax `a`, store packed codes, return this thread's residual sum.
template <bool WANT_RES>
__device__ __forceinline__ double quantize_cached_row(const Pack16 *v, int nchunk, float a,
                                                      uint32_t *__restrict__ qrow, float &s_out)
{
    float s = 1.0f, inv = 0.0f;
    if (a != 0.0f) { s = a / 7.0f; inv = 7.0f / a; }
    s_out = s;
    double rs = 0.0;
#pragma unroll
    for (int r = 0; r < ROW_MAXCHUNK; ++r) {
        int c = threadIdx.x + ROW_THREADS * r;
        if (c < nchunk) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f = (float)v[r].h[e];
                int code = code_from(rintf(f * inv));
                word |= (uint32_t)(code & 0xF) << (4 * e);
                if (WANT_RES) {
                    float deq = (float)code * s;
                    float rr = deq - f;
                    rs += (double)rr * (double)rr;
                }
            }
            if (qrow) qrow[c] = word;
        }
    }
    return rs;
}

