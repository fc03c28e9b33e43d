// Pieces shared by the W4A4 GEMM kernels: the int4 -> int8 unpack and the XCD-aware tile order.
#pragma once
#include "common.h"

// A nibble placed in the HIGH half of a byte is the int8 value 16*code (two's complement carries
// the sign), so "(w << 4) & 0xF0F0F0F0" and "w & 0xF0F0F0F0" turn one packed dword into two dwords
// of int8 without any sign-extension arithmetic: lo holds the even elements, hi the odd ones.
__device__ __forceinline__ void unpack16(const uint4 &v, uint4 &lo, uint4 &hi)
{
    lo.x = (v.x << 4) & 0xF0F0F0F0u; hi.x = v.x & 0xF0F0F0F0u;
    lo.y = (v.y << 4) & 0xF0F0F0F0u; hi.y = v.y & 0xF0F0F0F0u;
    lo.z = (v.z << 4) & 0xF0F0F0F0u; hi.z = v.z & 0xF0F0F0F0u;
    lo.w = (v.w << 4) & 0xF0F0F0F0u; hi.w = v.w & 0xF0F0F0F0u;
}
__device__ __forceinline__ i32x4 as_i32x4(const uint4 &t)
{
    return i32x4{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
}

// XCD-aware tile id: consecutive dispatch ids go round-robin over the 8 XCDs
// (each with its own L2), so give each XCD a contiguous range of tiles.
__device__ __forceinline__ int xcd_remap(int pid, int total)
{
    int x = pid & 7, idx = pid >> 3;
    int per = total >> 3, rem = total & 7;
    return x * per + (x < rem ? x : rem) + idx;
}
