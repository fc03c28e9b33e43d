// Shared device helpers for the gfx950 kernels of libquota (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include "../../include/quota.h"
#include "profile.h"

#define QUOTA_WAVE 64

// launch-error check used by every host entry point after it enqueues kernels
#define QUOTA_RETURN_IF_LAUNCH_FAILED()                    \
    do {                                                   \
        if (hipGetLastError() != hipSuccess) return QUOTA_ERR_HIP; \
    } while (0)

typedef _Float16 f16;
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

union Pack16 {           // 16 bytes seen as halves, dwords or one vector load
    uint4 u;
    f16 h[8];
    uint32_t w[4];
};

// Wave-wide reductions with DPP moves (no LDS crossbar): an inclusive scan -- shifts by 1, 2, 4, 8
// inside each row of 16 lanes, then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into
// rows 2 and 3 -- leaves the result of all 64 lanes in lane 63, which is read back as a scalar.
// Lanes without a source combine with the operation's identity.
#define QUOTA_DPP_STEPS(STEP) \
    STEP(0x111, 0xf) STEP(0x112, 0xf) STEP(0x114, 0xf) STEP(0x118, 0xf) STEP(0x142, 0xa) STEP(0x143, 0xc)

__device__ __forceinline__ float wave_max(float v)
{
#define STEP(ctrl, rows)                                                                              \
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), ctrl, \
                                                            rows, 0xf, false)));
    QUOTA_DPP_STEPS(STEP)
#undef STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ double wave_sum(double v)
{
#define STEP(ctrl, rows)                                                                       \
    {                                                                                          \
        const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), ctrl, rows, 0xf, false); \
        const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), ctrl, rows, 0xf, false); \
        v += __hiloint2double(hi, lo);                                                         \
    }
    QUOTA_DPP_STEPS(STEP)
#undef STEP
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63),
                            __builtin_amdgcn_readlane(__double2loint(v), 63));
}
__device__ __forceinline__ float wave_sum(float v)
{
#define STEP(ctrl, rows) \
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, rows, 0xf, false));
    QUOTA_DPP_STEPS(STEP)
#undef STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// block-wide (blockDim.x = 64*NW) max of a float and sum of up to two doubles;
// every thread gets the result.  `sm` needs 3*NW doubles of LDS.
template <int NW>
__device__ __forceinline__ void block_max_sum2(float &mx, double &s0, double &s1, double *sm)
{
    mx = wave_max(mx);
    s0 = wave_sum(s0);
    s1 = wave_sum(s1);
    int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    __syncthreads();          // protect sm against the previous use
    if (l == 0) { sm[w] = (double)mx; sm[NW + w] = s0; sm[2 * NW + w] = s1; }
    __syncthreads();
    float m = (float)sm[0];
    double a = sm[NW], b = sm[2 * NW];
#pragma unroll
    for (int i = 1; i < NW; ++i) { m = fmaxf(m, (float)sm[i]); a += sm[NW + i]; b += sm[2 * NW + i]; }
    mx = m; s0 = a; s1 = b;
}

// fp32 -> fp16 with the fp32 value materialised first.  Without the barrier
// the compiler may fold "multiply/add, then convert" into one mixed-precision
// instruction that rounds the exact result straight to fp16; the two-step
// rounding written here is what the rest of the pipeline is defined with.
__device__ __forceinline__ f16 to_f16(float v)
{
    asm volatile("" : "+v"(v));
    return (f16)v;
}

// int4 code from a rounded fp32 value: clamp to [-8, 7]
__device__ __forceinline__ int code_from(float r)
{
    r = fminf(fmaxf(r, -8.0f), 7.0f);
    return (int)r;
}

// The int4 code of a scaled value t = x * (7 / absmax), without a round / convert / mask chain:
// clamp to [-8, 7] first (the bounds are integers, so clamping commutes with rounding to integer),
// then add 1.5 * 2^23 -- in that binade one unit in the last place is 1, so the fp32 add itself
// rounds to the nearest integer, ties to even, and the low mantissa bits of the sum hold the code in
// two's complement.  code_bits(t) & 0xF is the packed nibble; code_float(bits) the code as a float.
#define ROW_MAGIC 12582912.0f
__device__ __forceinline__ uint32_t code_bits(float t)
{
    t = fminf(fmaxf(t, -8.0f), 7.0f);          // NaN -> -8, as in code_from
    return __float_as_uint(t + ROW_MAGIC);
}
__device__ __forceinline__ float code_float(uint32_t bits) { return __uint_as_float(bits) - ROW_MAGIC; }

