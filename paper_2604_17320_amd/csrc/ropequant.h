// RoPE and the 4-bit K/V group quantizer on one 8-channel chunk, shared by the stand-alone
// RoPE/KV kernel and the fused epilogue of the QKV GEMM (both must round identically).
#pragma once
#include "common.h"

// Quantize this lane's 8 channels; the 8 lanes [lane & ~7, +8) form one 64-channel group and
// must all call this together.  Returns packed codes; *sh_out = fp16 group scale; xhat
// (optional) = fp16(code * scale), the value attention sees.
__device__ __forceinline__ uint32_t kv_quant8(const float f[8], f16 *sh_out, Pack16 *xhat)
{
    float a = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf(f[e]));
    a = fmaxf(a, __shfl_xor(a, 1, 64));
    a = fmaxf(a, __shfl_xor(a, 2, 64));
    a = fmaxf(a, __shfl_xor(a, 4, 64));
    f16 sh = to_f16(a / 7.0f);
    float s = (float)sh;
    if (a == 0.0f || s == 0.0f) { sh = (f16)1.0f; s = 1.0f; }
    float r = 1.0f / s;
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t cb = code_bits(f[e] * r);
        word |= (cb & 0xFu) << (4 * e);
        if (xhat) xhat->h[e] = to_f16(code_float(cb) * s);
    }
    *sh_out = sh;
    return word;
}

// Rotate-half RoPE of one chunk: x holds channels [8c, 8c+8) of a head, xp the partner chunk
// half a head away, cs / sn the angle table entries of these 8 pair indices; `second` says
// whether x lies in the second half of the head.  fp32 products, one add, rounded to fp16.
__device__ __forceinline__ void rope8(const Pack16 &x, const Pack16 &xp, const float cs[8],
                                      const float sn[8], bool second, Pack16 &out)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float a = (float)x.h[e] * cs[e];
        float b = (float)xp.h[e] * sn[e];
        out.h[e] = to_f16(second ? a + b : a - b);
    }
}
