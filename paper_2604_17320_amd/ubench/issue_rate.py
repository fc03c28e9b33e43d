#!/usr/bin/env python3
"""Issue-rate probe for gfx950: what one v_mfma_i32_32x32x32_i8 and one fp32 vector instruction cost
a SIMD's issue, alone and interleaved, at one and two waves per SIMD.

The W4A4 GEMM needs, per 32x32x32 MFMA, 8 vector instructions for the per-group fp32 scale (one
convert + one fma per output element and 128-deep group) and about 6 more to unpack int4 operands.
This probe places exactly that mix by hand (one asm block, fixed registers, register-to-register
only, no memory access in the timed loop, results meaningless) so that the compiler's scheduling is
out of the picture, and prints ns per block of 16 MFMAs.

    python -m paper_2604_17320_amd.ubench.issue_rate        # needs hipcc and a GPU
"""
import os
import subprocess
import sys
import tempfile

TEMPLATE = r'''
#include <hip/hip_runtime.h>
#include <cstdio>
template <int MODE>
__global__ __launch_bounds__(256) void k(float *out, int iters)
{
    float s = threadIdx.x;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
        if (MODE == 0) asm volatile("@@M@@" ::: @@CLOB@@);
        else if (MODE == 1) asm volatile("@@V@@" ::: @@CLOB@@);
        else if (MODE == 2) asm volatile("@@B8@@" ::: @@CLOB@@);
        else asm volatile("@@B14@@" ::: @@CLOB@@);
    }
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
template <int MODE>
void run(const char *what, float *d, int wgs)
{
    const int iters = 4000;
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    k<MODE><<<wgs, 256>>>(d, 10);
    (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0);
    k<MODE><<<wgs, 256>>>(d, iters);
    (void)hipEventRecord(e1);
    (void)hipEventSynchronize(e1);
    float ms; (void)hipEventElapsedTime(&ms, e0, e1);
    printf("%-44s workgroups=%4d (%d wave(s) per SIMD)  %7.1f ns per block\n", what, wgs, wgs / 256, ms * 1e6 / iters);
}
int main()
{
    float *d;
    if (hipMalloc(&d, 4096 * 256 * 4) != hipSuccess) return 2;
    for (int wgs : {256, 512}) {
        run<0>("16 MFMA", d, wgs);
        run<1>("128 VALU (64 x convert + fma)", d, wgs);
        run<2>("16 x (1 MFMA + 8 VALU)", d, wgs);
        run<3>("16 x (1 MFMA + 14 VALU)", d, wgs);
    }
    return 0;
}
'''


def block(with_mfma, chain, extra):
    """16 slots; per slot optionally one MFMA (two accumulator sets take turns, the vector work reads the
    other one), `chain` convert+fma pairs and `extra` integer instructions."""
    lines, accs = [], [(64, 79), (80, 95)]
    for t in range(4):
        a, p = accs[t & 1], accs[(t + 1) & 1]
        r = 0
        for k in range(4):
            if with_mfma:
                c = "0" if k == 0 else f"v[{a[0]}:{a[1]}]"
                lines.append(f"v_mfma_i32_32x32x32_i8 v[{a[0]}:{a[1]}], v[160:163], v[164:167], {c}")
            for _ in range(chain):
                lines.append(f"v_cvt_f32_i32_e32 v168, v{p[0] + r}")
                lines.append(f"v_fmac_f32_e32 v{96 + 16 * t + r}, v168, v169")
                r += 1
            for q in range(extra):
                reg = 170 + q % 8
                lines.append(f"v_and_b32_e32 v{reg}, 0xf0f0f0f0, v{reg}" if q % 3 else f"v_lshlrev_b32_e32 v{reg}, 4, v{reg}")
    return "\\n\\t".join(lines)


def main():
    src = (TEMPLATE.replace("@@M@@", block(True, 0, 0)).replace("@@V@@", block(False, 4, 0))
           .replace("@@B8@@", block(True, 4, 0)).replace("@@B14@@", block(True, 4, 6))
           .replace("@@CLOB@@", ",".join(f'"v{i}"' for i in range(64, 180))))
    with tempfile.TemporaryDirectory() as tmp:
        path, exe = os.path.join(tmp, "issue_rate.hip"), os.path.join(tmp, "issue_rate")
        with open(path, "w") as f:
            f.write(src)
        subprocess.run([os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O3", path, "-o", exe],
                       check=True)
        return subprocess.run([exe]).returncode


if __name__ == "__main__":
    sys.exit(main())
