"""GPU parity of the sensitivity profiling behind Eq. 1 against the oracle's fp64 profiler: the
full-precision block, the per-sample deviation norms, the block profile and the recipe that
follows from it.

Tolerances.  The library's full-precision block stores fp16 between its steps and accumulates in
fp32; the oracle's is plain fp64.  A block output therefore agrees element-wise within 1e-2 of
max(|value|, rms) (in practice a few fp16 ulps), the reference norm ||x|| within 1e-3 relative.
The deviation ||x^q - x|| is a difference of two block outputs of which the low-bit one is
bit-exact against the oracle (teacher-forced layer tests), so its error is the full-precision
block's fp16 noise (about 1e-3 of ||x||) against a deviation of about 1e-1 of ||x||: 1 % relative
is asserted, and the same for S."""
import numpy as np
import pytest
import torch

import oracle
from oracle import profiler as oprof
from paper_2604_17320_amd import workloads as wl
from test_gpu_ops import close_f16, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available()
    from paper_2604_17320_amd import binding
    binding.lib()
    return binding


def build_pair(d, H, Hkv, dh, F, n_pos, seed, scale=0.02):
    """One layer twice: fp16 weights for the full-precision block, and their int4 quantization for
    the deployed one, both as oracle structures and as device layers."""
    from paper_2604_17320_amd.model import FullPrecisionLayer, PackedLinear, PrefillLayer
    r = wl.rng(seed, "profiler")
    dq = (H + 2 * Hkv) * dh
    fw = {name: (r.standard_normal(shp, dtype=np.float32) * np.float32(scale)).astype(np.float16)
          for name, shp in dict(qkv=(dq, d), o=(d, d), gu=(2 * F, d), down=(d, F)).items()}
    g1 = r.uniform(0.7, 1.3, d).astype(np.float32)
    g2 = r.uniform(0.7, 1.3, d).astype(np.float32)
    q = {k: oracle.quantize_weights(v.astype(np.float32)) for k, v in fw.items()}
    Wq = oracle.LayerWeights(qkv=q["qkv"], o=q["o"], gu=q["gu"], down=q["down"], gamma1=g1, gamma2=g2,
                             eps=1e-5, H=H, dh=dh, F=F, Hkv=Hkv)
    Wf = oprof.FullPrecisionWeights(qkv=fw["qkv"], o=fw["o"], gu=fw["gu"], down=fw["down"], gamma1=g1, gamma2=g2,
                                    eps=1e-5, H=H, dh=dh, F=F, Hkv=Hkv)
    cos, sin = wl.rope_tables(dh, n_pos)
    lin = {k: PackedLinear.from_codes(dev(c), dev(s)) for k, (c, s) in q.items()}
    Lq = PrefillLayer(H, dh, F, lin["qkv"], lin["o"], lin["gu"], lin["down"], dev(g1), dev(g2), 1e-5,
                      dev(cos), dev(sin), Hkv=Hkv)
    Lf = FullPrecisionLayer(H, dh, F, dev(fw["qkv"]), dev(fw["o"]), dev(fw["gu"]), dev(fw["down"]), dev(g1),
                            dev(g2), 1e-5, dev(cos), dev(sin), Hkv=Hkv)
    return Wq, Wf, Lq, Lf, cos, sin


def inputs(B, N, d, seed, n_outlier=4):
    r = wl.rng(seed, "profiler-x")
    x = r.standard_normal((B * N, d), dtype=np.float32)
    x[:, r.permutation(d)[:n_outlier]] *= 20.0
    pos = np.tile(3 + 2 * np.arange(N, dtype=np.int32), B)
    return x.astype(np.float16), pos


CASES = [  # d, H, Hkv, dh, F, B, N
    (512, 8, 8, 64, 1376, 2, 80),        # the small layer; 160 rows = one full and one ragged row tile
    (512, 8, 2, 64, 1376, 3, 47),        # grouped K/V heads, odd sequence length
    (1024, 8, 4, 128, 2752, 1, 200),     # head_dim 128
]


@pytest.mark.parametrize("d,H,Hkv,dh,F,B,N", CASES)
def test_fp_block_against_oracle(qb, d, H, Hkv, dh, F, B, N):
    Wq, Wf, Lq, Lf, cos, sin = build_pair(d, H, Hkv, dh, F, 2 * N + 8, seed=d + N)
    x, pos = inputs(B, N, d, seed=N)
    want = oprof.block_full_precision(Wf, x, pos, B, N, cos, sin)
    got = host(Lf.forward(dev(x), dev(pos), B, N)).astype(np.float64)
    err = np.abs(got - want)
    print("max |err| / rms", err.max() / np.sqrt((want ** 2).mean()))
    assert close_f16(got, want)
    assert abs(np.linalg.norm(got) / np.linalg.norm(want) - 1.0) < 1e-3


def test_activation_deviation_against_oracle(qb):
    r = np.random.default_rng(5)
    B, n = 5, 3 * 1000 + 7                       # not a multiple of the workgroup size
    a = r.standard_normal((B, n)).astype(np.float16)
    b = (a.astype(np.float32) + 0.05 * r.standard_normal((B, n))).astype(np.float16)
    b[3] = a[3]                                  # one sample without any deviation
    dn = torch.empty(B, dtype=torch.float64, device="cuda")
    rn = torch.empty(B, dtype=torch.float64, device="cuda")
    qb.quota_activation_deviation(dev(b), dev(a), B, n, dn, rn)
    wd, wr = oprof.activation_deviation(b, a, B)
    assert np.allclose(host(dn), wd, rtol=1e-12, atol=0) and np.allclose(host(rn), wr, rtol=1e-12, atol=0)
    assert host(dn)[3] == 0.0


@pytest.mark.parametrize("d,H,Hkv,dh,F,B,N", CASES)
def test_profile_block_against_oracle(qb, d, H, Hkv, dh, F, B, N):
    from paper_2604_17320_amd.model import profile_sensitivity
    Wq, Wf, Lq, Lf, cos, sin = build_pair(d, H, Hkv, dh, F, 2 * N + 8, seed=d + N + 1)
    x, pos = inputs(B, N, d, seed=N + 1)
    S, dn, rn = profile_sensitivity(Lq, Lf, dev(x), dev(pos), B, N)
    wd, wr = oprof.profile_block(Wq, Wf, x, pos, B, N, 0, N - 8, cos, sin)
    wS = oracle.recipe.sensitivity(wd, wr, 1e-6)
    print("S", S, "oracle", wS, "diff_norm", dn, wd, "ref_norm", rn, wr)
    assert np.allclose(rn, wr, rtol=1e-3, atol=0)
    assert np.allclose(dn, wd, rtol=1e-2, atol=0)
    assert abs(S / wS - 1.0) < 1e-2 and 0.02 < S < 0.6


def test_profile_block_errors_and_scratch_cache(qb):
    from paper_2604_17320_amd.model import KVCache4
    d, H, Hkv, dh, F, B, N = CASES[0]
    Wq, Wf, Lq, Lf, cos, sin = build_pair(d, H, Hkv, dh, F, 2 * N + 8, seed=1)
    _, _, _, Lf_other, _, _ = build_pair(d, H, 2, dh, F, 2 * N + 8, seed=2)
    x, pos = inputs(B, N, d, seed=1)
    xd, pd = dev(x), dev(pos)
    dn = torch.empty(B, dtype=torch.float64, device="cuda")
    rn = torch.empty(B, dtype=torch.float64, device="cuda")
    ws = torch.empty(qb.quota_profile_block_workspace_bytes(Lq.desc, Lf.desc, B, N), dtype=torch.uint8, device="cuda")
    cache = KVCache4(B, N + 5, Hkv, dh)
    cache.desc.len = 5
    qb.quota_profile_block(Lq.desc, Lf.desc, xd, pd, B, N, cache.desc, dn, rn, ws)
    assert cache.len == 5                                          # handed back as it came
    with pytest.raises(qb.QuotaError) as e:                        # K/V head counts differ
        qb.quota_profile_block(Lq.desc, Lf_other.desc, xd, pd, B, N, cache.desc, dn, rn, ws)
    assert e.value.code == qb.ERR_SHAPE
    small = KVCache4(B, N - 1, Hkv, dh)                            # no room for the block's N rows
    with pytest.raises(qb.QuotaError) as e:
        qb.quota_profile_block(Lq.desc, Lf.desc, xd, pd, B, N, small.desc, dn, rn, ws)
    assert e.value.code == qb.ERR_CAPACITY and small.len == 0


def test_recipe_from_profiled_sensitivities(qb):
    """The whole offline path on synthetic calibration data: profile m candidate layers (different
    weights each, weight scale growing with depth so that the layers differ in sensitivity), then
    Eq. 2-5.  The keep ratios follow the oracle's recipe from the oracle's own profile."""
    from paper_2604_17320_amd.model import profile_sensitivity
    d, H, Hkv, dh, F, B, N = 512, 8, 8, 64, 1376, 4, 48
    S_gpu, S_orc = [], []
    for layer in range(5):
        Wq, Wf, Lq, Lf, cos, sin = build_pair(d, H, Hkv, dh, F, 2 * N + 8, seed=100 + layer, scale=0.01 * (1 + layer))
        x, pos = inputs(B, N, d, seed=200 + layer)
        S, _, _ = profile_sensitivity(Lq, Lf, dev(x), dev(pos), B, N)
        S_gpu.append(S)
        S_orc.append(oprof.profile_sensitivity(Wq, Wf, x, pos, B, N, 0, N - 8, cos, sin))
    print("S gpu", S_gpu, "oracle", S_orc)
    assert np.allclose(S_gpu, S_orc, rtol=1e-2)
    got = qb.quota_make_recipe(S_gpu, 1.0, 0.3, 576)
    want = oracle.recipe.make_recipe(S_orc, 1.0, 0.3, 576)
    assert np.allclose(got["r"], want["r"], atol=2e-2)
    assert np.all(np.abs(np.array(got["K"]) - np.array(want["K"])) <= 12)      # 2e-2 of 576
    assert all(a >= b for a, b in zip(got["K"], got["K"][1:]))


def test_profile_block_7b_shape(qb):
    """One block at the 7B shape (d = 4096, 32 heads, F = 11008), two samples of 576 + 64 tokens."""
    d, H, Hkv, dh, F, B, N = 4096, 32, 32, 128, 11008, 2, 640
    from paper_2604_17320_amd.model import profile_sensitivity
    Wq, Wf, Lq, Lf, cos, sin = build_pair(d, H, Hkv, dh, F, 2 * N + 8, seed=7)
    x, pos = inputs(B, N, d, seed=7, n_outlier=41)
    S, dn, rn = profile_sensitivity(Lq, Lf, dev(x), dev(pos), B, N)
    wd, wr = oprof.profile_block(Wq, Wf, x, pos, B, N, 0, 576, cos, sin)
    wS = oracle.recipe.sensitivity(wd, wr, 1e-6)
    print("S", S, "oracle", wS)
    assert np.allclose(rn, wr, rtol=1e-3, atol=0) and np.allclose(dn, wd, rtol=1e-2, atol=0)
    assert abs(S / wS - 1.0) < 1e-2
