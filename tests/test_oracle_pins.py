"""Pins for the CPU oracle (no GPU): every oracle function is checked against
something other than itself -- values the paper prints, closed forms,
invariants, brute force on tiny inputs, or a library routine for the special
case that reduces to one."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl


def R(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ fp16
def test_f16_to_f32_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    got = oracle.f16_to_f32(h)
    want = h.astype(np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_f64_to_f16_rounding_matches_ieee():
    r = R(1)
    x = np.concatenate([
        r.standard_normal(20000) * 10.0 ** r.uniform(-9, 5, 20000),
        # exact ties between neighbouring fp16 values, and subnormal range
        (np.arange(1, 4000, dtype=np.float64) + 0.5) * 2.0 ** -24,
        (np.arange(1024, 2048, dtype=np.float64) + 0.5) * 2.0 ** -3,
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -25, 2.0 ** -26]),
    ])
    got = oracle.f64_to_f16(x)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


# ------------------------------------------------------- weight quantizer
def test_weight_quant_range_roundtrip_and_bruteforce():
    w = (R(2).standard_normal((24, 384)) * 0.02).astype(np.float32)
    codes, scales = oracle.quantize_weights(w)
    assert codes.min() >= -8 and codes.max() <= 7
    s = np.repeat(scales.astype(np.float64), 128, axis=1)
    err = np.abs(w.astype(np.float64) - codes * s)
    assert np.all(err <= s / 2 * (1 + 1e-6))
    # scale is absmax/7 rounded to fp16 (relative 2^-11) per (row, group)
    amax = np.abs(w).reshape(24, 3, 128).max(axis=2)
    assert np.allclose(scales.astype(np.float64), amax / 7.0, rtol=2.0 ** -10, atol=0)
    # brute force: nearest of the 16 levels in fp64 (skip exact midpoints)
    levels = np.arange(-8, 8)[None, None, :]
    dist = np.abs(w.astype(np.float64)[..., None] - levels * s[..., None])
    best = dist.argmin(axis=2) - 8
    two = np.sort(dist, axis=2)[..., :2]
    clear = (two[..., 1] - two[..., 0]) > 1e-7 * s
    assert np.array_equal(codes[clear], best[clear]) and clear.mean() > 0.999


def test_weight_quant_ragged_last_group_equals_zero_padding():
    w = (R(3).standard_normal((5, 1376)) * 0.02).astype(np.float32)   # 10*128 + 96
    c, s = oracle.quantize_weights(w)
    wp = np.zeros((5, 1408), np.float32)
    wp[:, :1376] = w
    cp, sp = oracle.quantize_weights(wp)
    assert s.shape == (5, 11)
    assert np.array_equal(s, sp) and np.array_equal(c, cp[:, :1376]) and not cp[:, 1376:].any()


def test_weight_quant_zero_group_and_scale_invariance():
    w = (R(4).standard_normal((3, 256)) * 0.02).astype(np.float32)
    w[1, 128:] = 0.0
    c, s = oracle.quantize_weights(w)
    assert s[1, 1] == np.float16(1.0) and not c[1, 128:].any()
    c2, s2 = oracle.quantize_weights(w * 2.0)
    assert np.array_equal(c2, c)
    assert np.array_equal(s2[s != 1.0].astype(np.float32), 2 * s[s != 1.0].astype(np.float32))


# ---------------------------------------------------- activation quantizer
def test_act_quant_invariants():
    x = wl.hidden_state(wl.CONFIGS[0], seed=5)
    q, s, ss, rs = oracle.quantize_act(x)
    xd = x.astype(np.float64)
    assert q.min() >= -8 and q.max() <= 7
    assert np.allclose(s, np.abs(xd).max(axis=1) / 7.0, rtol=1e-6)
    err = np.abs(xd - q * s[:, None].astype(np.float64))
    assert np.all(err <= s[:, None] / 2 * (1 + 2.0 ** -20))
    assert np.allclose(ss, (xd ** 2).sum(axis=1), rtol=1e-7)
    assert np.allclose(rs, (err ** 2).sum(axis=1), rtol=1e-5)
    assert np.all(np.sqrt(rs) <= s / 2 * math.sqrt(x.shape[1]) * (1 + 1e-6))
    # brute force nearest level
    sd = s[:, None, None].astype(np.float64)
    dist = np.abs(xd[..., None] - np.arange(-8, 8)[None, None, :] * sd)
    two = np.sort(dist, axis=2)[..., :2]
    clear = (two[..., 1] - two[..., 0]) > 1e-5 * sd[..., 0]
    assert np.array_equal(q[clear], (dist.argmin(axis=2) - 8)[clear]) and clear.mean() > 0.99


def test_act_quant_scaling_zero_row_and_grid():
    x = wl.hidden_state(wl.CONFIGS[0], seed=6)[:8]
    x[3] = 0
    q, s, ss, rs = oracle.quantize_act(x)
    assert s[3] == 1.0 and not q[3].any() and ss[3] == 0 and rs[3] == 0
    q2, s2, _, _ = oracle.quantize_act(x * np.float16(2))
    keep = np.arange(8) != 3
    assert np.array_equal(q2, q) and np.array_equal(s2[keep], 2 * s[keep])
    # vectors already on the int4 grid (step 0.5, max |code| 7) have zero residual
    codes = R(7).integers(-7, 8, size=(4, 256))
    codes[:, 0] = 7
    g = (codes * 0.5).astype(np.float16)
    qg, sg, ssg, rsg = oracle.quantize_act(g)
    assert np.array_equal(qg, codes) and np.all(sg == 0.5) and np.all(rsg == 0)
    assert np.array_equal(ssg, ((codes * 0.5) ** 2).sum(axis=1).astype(np.float32))


# ------------------------------------------------------------------ GEMM
def test_gemm_matches_fp64_matmul_of_dequantized_operands():
    r = R(8)
    M, K, N = 7, 1376, 13        # ragged last group, all three sizes distinct
    qa = r.integers(-8, 8, (M, K)).astype(np.int8)
    sa = r.uniform(0.1, 2.0, M).astype(np.float32)
    w = (r.standard_normal((N, K)) * 0.02).astype(np.float32)
    qw, sw = oracle.quantize_weights(w)
    res = r.standard_normal((M, N)).astype(np.float16)
    y, acc = oracle.w4a4_gemm(qa, sa, qw, sw, want_acc=True)
    yr = oracle.w4a4_gemm(qa, sa, qw, sw, residual=res)
    swf = np.repeat(sw.astype(np.float64), 128, axis=1)[:, :K]
    ref = (qa.astype(np.float64) * sa[:, None]) @ (qw.astype(np.float64) * swf).T
    assert np.array_equal(acc, qa.astype(np.int64) @ qw.astype(np.int64).T)
    tol = 2.0 ** -10
    assert np.allclose(y.astype(np.float64), ref, rtol=tol, atol=1e-4)
    assert np.allclose(yr.astype(np.float64), ref + res.astype(np.float64), rtol=tol, atol=2e-3)


def test_gemm_unit_scales_and_identity_weights():
    r = R(9)
    M, K = 5, 256
    qa = r.integers(-8, 8, (M, K)).astype(np.int8)
    sa = np.ones(M, np.float32)
    qw = r.integers(-8, 8, (6, K)).astype(np.int8)
    sw = np.ones((6, 2), np.float16)
    y, acc = oracle.w4a4_gemm(qa, sa, qw, sw, want_acc=True)
    exact = qa.astype(np.int64) @ qw.astype(np.int64).T
    assert np.array_equal(acc, exact)
    assert np.array_equal(y, exact.astype(np.float16))       # |sum| < 2^14, one rounding
    # weight rows that pick a single channel with code 7 and scale 0.25
    qi = np.zeros((K, K), np.int8)
    qi[np.arange(K), np.arange(K)] = 7
    si = np.full((K, 2), 0.25, np.float16)
    sa2 = r.uniform(0.5, 1.5, M).astype(np.float32)
    yi = oracle.w4a4_gemm(qa, sa2, qi, si)
    want = (qa.astype(np.float32) * np.float32(1.75) * sa2[:, None]).astype(np.float16)
    assert np.array_equal(yi, want)


def test_gemm_group_scales_are_per_group():
    # one group carries all the signal: y = sa * sw[n, g] * acc_g exactly
    K = 384
    qa = np.zeros((1, K), np.int8)
    qa[0, 128:256] = 3
    qw = np.full((2, K), 2, np.int8)
    sw = np.array([[1, 0.5, 4], [2, 0.125, 8]], np.float16)
    y = oracle.w4a4_gemm(qa, np.array([0.5], np.float32), qw, sw)
    assert np.array_equal(y, np.array([[0.5 * 0.5 * 768, 0.5 * 0.125 * 768]], np.float16))


# ------------------------------------------------------------------ RoPE
def test_rope_identity_quarter_turn_and_relative_property():
    r = R(10)
    H, dh, M = 2, 64, 6
    x = r.standard_normal((M, H * dh)).astype(np.float16)
    cos, sin = wl.rope_tables(dh, 64)
    pos0 = np.zeros(M, np.int32)
    assert np.array_equal(oracle.rope(x, H, dh, pos0, cos, sin), x)
    # a table entry with cos = 0, sin = 1 turns (x1, x2) into (-x2, x1)
    c1 = np.zeros((1, dh // 2), np.float32)
    s1 = np.ones((1, dh // 2), np.float32)
    y = oracle.rope(x, H, dh, pos0, c1, s1).reshape(M, H, 2, dh // 2)
    xr = x.reshape(M, H, 2, dh // 2)
    assert np.array_equal(y[:, :, 0], -xr[:, :, 1]) and np.array_equal(y[:, :, 1], xr[:, :, 0])
    # rotation preserves each pair's norm and q.k depends on p - p' only
    pos = np.array([3, 10, 17, 30, 40, 63], np.int32)
    y = oracle.rope(x, H, dh, pos, cos, sin).astype(np.float64).reshape(M, H, 2, dh // 2)
    n_in = (xr.astype(np.float64) ** 2).sum(axis=2)
    assert np.allclose((y ** 2).sum(axis=2), n_in, rtol=4e-3, atol=1e-5)
    a = np.tile(x[:1], (2, 1))
    b = np.tile(x[1:2], (2, 1))
    ra = oracle.rope(a, H, dh, np.array([5, 25], np.int32), cos, sin).astype(np.float64)
    rb = oracle.rope(b, H, dh, np.array([12, 32], np.int32), cos, sin).astype(np.float64)
    d = (ra * rb).reshape(2, H, dh).sum(axis=2)
    assert np.allclose(d[0], d[1], atol=0.05)


# -------------------------------------------------------------- KV quant
def test_kv_quant_invariants():
    r = R(11)
    x = (r.standard_normal((9, 256)) * 3).astype(np.float16)
    x[2, 64:128] = 0
    c, s, xh = oracle.kv_quant(x)
    assert c.min() >= -8 and c.max() <= 7 and s.shape == (9, 4)
    sd = np.repeat(s.astype(np.float64), 64, axis=1)
    assert np.all(np.abs(x.astype(np.float64) - c * sd) <= sd / 2 * (1 + 2e-3))
    assert np.array_equal(xh, (c * sd).astype(np.float16))
    assert s[2, 1] == np.float16(1) and not c[2, 64:128].any()
    assert np.allclose(s.astype(np.float64)[s != 1], (np.abs(x).reshape(9, 4, 64).max(axis=2) / 7.0)[s != 1],
                       rtol=2.0 ** -10)
    c2, s2, _ = oracle.kv_quant(x * np.float16(2))
    assert np.array_equal(c2, c)
    # groups are independent
    x3 = x.copy()
    x3[:, :64] *= np.float16(0.5)
    c3, s3, _ = oracle.kv_quant(x3)
    assert np.array_equal(c3[:, 64:], c[:, 64:]) and np.array_equal(s3[:, 1:], s[:, 1:])


# ------------------------------------------------------------- attention
def _small_qkv(seed, B, N, H, dh):
    r = R(seed)
    q = r.standard_normal((B * N, H * dh)).astype(np.float16)
    k = r.standard_normal((B * N, H * dh)).astype(np.float16)
    v = r.standard_normal((B * N, H * dh)).astype(np.float16)
    return q, k, v


@pytest.mark.parametrize("vis_begin,Nv", [(0, 6), (2, 5)])
def test_attention_matches_library_sdpa_and_column_sums(vis_begin, Nv):
    B, N, H, dh = 2, 10, 3, 16
    q, k, v = _small_qkv(12, B, N, H, dh)
    o, ci, cv, P = oracle.attention(q, k, v, B, N, H, dh, vis_begin, Nv, want_P=True)
    t = lambda a: torch.from_numpy(a.astype(np.float64)).reshape(B, N, H, dh).permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(t(q), t(k), t(v), is_causal=True)
    ref = ref.permute(0, 2, 1, 3).reshape(B * N, H * dh).numpy()
    assert np.allclose(o.astype(np.float64), ref, rtol=2.0 ** -10, atol=1e-6)
    assert np.allclose(P.sum(axis=3), 1.0, atol=1e-12)
    assert np.all(np.triu(P, 1) == 0)
    vis = np.zeros(N, bool)
    vis[vis_begin:vis_begin + Nv] = True
    Pm = P.mean(axis=1)                                    # [B, query, key]
    assert np.allclose(ci, Pm[:, ~vis][:, :, vis].sum(axis=1), rtol=1e-6)
    assert np.allclose(cv, Pm[:, vis][:, :, vis].sum(axis=1), rtol=1e-6)
    # all column masses over all keys sum to the number of query rows
    total_text = Pm[:, ~vis].sum()
    assert np.isclose(ci.sum() + Pm[:, ~vis][:, :, ~vis].sum(), total_text)
    assert np.isclose(total_text, B * (N - Nv))


def test_attention_uniform_logits_closed_form():
    B, N, H, dh = 1, 12, 2, 8
    _, k, v = _small_qkv(13, B, N, H, dh)
    q = np.zeros((N, H * dh), np.float16)
    vis_begin, Nv = 3, 6
    o, ci, cv = oracle.attention(q, k, v, B, N, H, dh, vis_begin, Nv)
    assert np.array_equal(o[0], v[0])                       # first token sees itself only
    run = np.cumsum(v.astype(np.float64), axis=0) / np.arange(1, N + 1)[:, None]
    assert np.allclose(o.astype(np.float64), run, rtol=2.0 ** -10, atol=1e-6)
    inv = 1.0 / np.arange(1, N + 1)
    for i in range(Nv):
        key = vis_begin + i
        # queries at or after the key, by class; text before the image sees no visual key
        intra = inv[key:vis_begin + Nv].sum()
        inter = inv[vis_begin + Nv:].sum()
        assert np.isclose(cv[0, i], intra, rtol=1e-6) and np.isclose(ci[0, i], inter, rtol=1e-6)


# --------------------------------------------------------------- scoring
def _metrics(seed, B, Nv):
    r = R(seed)
    return (r.uniform(1, 9, (B, Nv)).astype(np.float32), r.uniform(0.1, 2, (B, Nv)).astype(np.float32),
            r.uniform(0, 1, (B, Nv)).astype(np.float32), r.uniform(0, 3, (B, Nv)).astype(np.float32))


def test_score_normalisation_ranks_and_range():
    B, Nv = 2, 11
    ss, rs, ci, cv = _metrics(14, B, Nv)
    ci[0] = R(15).permutation(Nv).astype(np.float32)      # 0..10: ranks 1 and 9 -> lo=1, hi=9
    sc, g = oracle.score(ss, rs, ci, cv, want_normed=True)
    assert g.min() >= 0 and g.max() <= 1
    assert np.array_equal(g[1, 0], np.clip((ci[0] - 1) / np.float32(8), 0, 1).astype(np.float32))
    for k, m in enumerate([np.sqrt(ss), ci, cv, np.sqrt(rs)]):
        order = np.argsort(m, axis=1, kind="stable")
        for b in range(B):
            assert np.all(g[k, b, order[b, 9:]] == 1) and np.all(g[k, b, order[b, :2]] == 0)
            mid = g[k, b, order[b, 2:9]]
            assert np.all(np.diff(mid) >= 0) and np.all((mid >= 0) & (mid <= 1))
    assert sc.min() >= 0 and sc.max() <= 1 + 1e-6


def test_score_affine_invariance_flat_metric_and_single_weight():
    B, Nv = 1, 37
    ss, rs, ci, cv = _metrics(16, B, Nv)
    _, g = oracle.score(ss, rs, ci, cv, want_normed=True)
    _, g4 = oracle.score(ss, rs, ci * 4, cv * 0.5, want_normed=True)
    assert np.array_equal(g4, g)                            # power-of-two scaling is exact
    _, ga = oracle.score(ss, rs, ci * 3 + 5, cv, want_normed=True)
    assert np.allclose(ga[1], g[1], atol=2e-6)
    flat = np.full((B, Nv), 0.7, np.float32)
    _, gf = oracle.score(ss, rs, flat, cv, want_normed=True)
    assert np.all(gf[1] == 0.5)
    for k, w in enumerate([dict(w_m=1, w_c=0, w_s=0, w_r=0), dict(w_m=0, w_c=1, w_s=0, w_r=0),
                           dict(w_m=0, w_c=0, w_s=1, w_r=0), dict(w_m=0, w_c=0, w_s=0, w_r=1)]):
        assert np.array_equal(oracle.score(ss, rs, ci, cv, **w), g[k])
    # percentiles are parameters: 0/100 is plain min-max scaling
    _, gmm = oracle.score(ss, rs, ci, cv, p_lo=0, p_hi=100, want_normed=True)
    want = (ci - ci.min()) / (ci.max() - ci.min())
    assert np.array_equal(gmm[1], want.astype(np.float32))


def test_score_weight_vectors_from_table5(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "table5_metric_weights.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 9 and rows[0][0] == "default"
    ss, rs, ci, cv = _metrics(17, 1, 64)
    _, g = oracle.score(ss, rs, ci, cv, want_normed=True)
    for name, inter, mag, intra, quant in rows:
        w = np.array([float(mag), float(inter), float(intra), float(quant)]) / 100.0
        assert abs(w.sum() - 1.0) < 2e-4, name
        sc = oracle.score(ss, rs, ci, cv, w_m=w[0], w_c=w[1], w_s=w[2], w_r=w[3])
        ref = (w[:, None, None] * g.astype(np.float64)).sum(axis=0)
        assert np.allclose(sc, ref, atol=3e-7), name
    d = dict(zip(["w_c", "w_m", "w_s", "w_r"], [float(v) / 100 for v in rows[0][1:]]))
    assert d == oracle.DEFAULT_WEIGHTS


# ----------------------------------------------------------------- top-k
def test_topk_equals_full_sort_with_ties():
    r = R(18)
    B, Nv = 3, 97
    sc = np.round(r.uniform(0, 1, (B, Nv)) * 20).astype(np.float32) / 20    # many ties
    for K in [0, 1, 19, 29, 96, 97, 150]:
        idx = oracle.topk(sc, K)
        k = min(K, Nv)
        assert idx.shape == (B, k)
        for b in range(B):
            order = np.lexsort((np.arange(Nv), -sc[b]))      # score desc, index asc
            assert np.array_equal(idx[b], np.sort(order[:k]))
            assert len(set(idx[b].tolist())) == k
    assert np.array_equal(oracle.topk(np.ones((1, 9), np.float32), 4)[0], np.arange(4))
    assert np.array_equal(oracle.topk(sc, Nv)[1], np.arange(Nv))


def test_topk_exhaustive_small():
    r = R(19)
    for trial in range(30):
        n = int(r.integers(1, 9))
        K = int(r.integers(0, n + 1))
        sc = r.integers(0, 4, (1, n)).astype(np.float32)
        got = tuple(oracle.topk(sc, K)[0].tolist())
        best = max(itertools.combinations(range(n), K),
                   key=lambda c: (sum(sc[0, list(c)]), [-i for i in c]))
        # maximal score sum; among equal sums the lexicographically smallest index set
        assert got == best


def test_budget_from_table4(golden_dir):
    for line in open(os.path.join(golden_dir, "budget_table4.txt")):
        if line.startswith("#") or not line.strip():
            continue
        V0, r, K = line.split()
        assert oracle.budget(float(r), int(V0)) == int(K)
    assert oracle.budget(0.3, 64) == 20 and oracle.budget(1.0, 576) == 576 and oracle.budget(0.0, 576) == 0


# ---------------------------------------------------- SwiGLU and RMSNorm
def test_silu_mul_against_library():
    r = R(20)
    gu = (r.standard_normal((5, 64)) * 4).astype(np.float16)
    gu[0, 0] = 0
    gu[0, 1] = -60
    z = oracle.silu_mul(gu, 32)
    t = torch.from_numpy(gu.astype(np.float64))
    ref = (torch.nn.functional.silu(t[:, :32]) * t[:, 32:]).numpy()
    assert np.array_equal(z, ref.astype(np.float16))
    assert z[0, 0] == 0 and abs(float(z[0, 1])) == 0


def test_rmsnorm_against_library():
    r = R(21)
    x = (r.standard_normal((6, 96)) * 3).astype(np.float16)
    gamma = r.uniform(0.5, 1.5, 96).astype(np.float32)
    h = oracle.rmsnorm(x, gamma, 1e-5)
    t = torch.from_numpy(x.astype(np.float64))
    ref = torch.nn.functional.rms_norm(t, (96,), torch.from_numpy(gamma.astype(np.float64)), eps=1e-5).numpy()
    assert np.allclose(h.astype(np.float64), ref, rtol=2.0 ** -10, atol=1e-7)
    h1 = oracle.rmsnorm(x, np.ones(96, np.float32), 0.0)
    assert np.allclose((h1.astype(np.float64) ** 2).mean(axis=1), 1.0, rtol=2e-3)
    assert np.array_equal(oracle.rmsnorm(x * np.float16(2), np.ones(96, np.float32), 0.0), h1)


# ------------------------------------------------------ layer composite
def _small_layer(seed=0, Nv=12, Nt=4, vis_begin=0):
    shape = wl.Shape("t", d=128, H=2, F=160, layers=1, B=2, Nv=Nv, Nt=Nt, n_outlier=2, vis_begin=vis_begin)
    fw = wl.fp_weights(shape, seed)
    W = oracle.LayerWeights(qkv=oracle.quantize_weights(fw["qkv"]), o=oracle.quantize_weights(fw["o"]),
                            gu=oracle.quantize_weights(fw["gu"]), down=oracle.quantize_weights(fw["down"]),
                            gamma1=np.ones(128, np.float32), gamma2=np.ones(128, np.float32),
                            eps=1e-5, H=2, dh=64, F=160)
    x = wl.hidden_state(shape, seed)
    pos = wl.positions(shape)
    cos, sin = wl.rope_tables(64, shape.N)
    return shape, W, x, pos, cos, sin


@pytest.mark.parametrize("vis_begin", [0, 2])
def test_layer_prune_mid_equals_prune_at_block_end(vis_begin):
    shape, W, x, pos, cos, sin = _small_layer(1, vis_begin=vis_begin)
    a = oracle.prefill_layer(W, x, pos, shape.B, shape.N, vis_begin, shape.Nv, 5, cos, sin)
    b = oracle.prefill_layer(W, x, pos, shape.B, shape.N, vis_begin, shape.Nv, 5, cos, sin, prune_mid=True)
    for key in ["x_next", "x1", "gu", "z", "qa4", "keep_idx", "pos_next", "cache_kc", "cache_vs"]:
        assert np.array_equal(a[key], b[key]), key


def test_layer_compaction_alignment():
    shape, W, x, pos, cos, sin = _small_layer(2, vis_begin=2)
    B, N, Nv, K = shape.B, shape.N, shape.Nv, 5
    out = oracle.prefill_layer(W, x, pos, B, N, 2, Nv, K, cos, sin)
    assert out["n_keep"] == K + shape.Nt and out["Nv_next"] == K
    assert out["cache_kc"].shape[0] == B * (K + shape.Nt)
    rows = out["rows"]
    for b in range(B):
        assert np.all(np.diff(rows[b]) > 0)
        txt = set(range(0, 2)) | set(range(2 + Nv, N))
        assert txt <= set(rows[b].tolist())
        p = out["pos_next"].reshape(B, -1)[b]
        assert np.array_equal(p, pos.reshape(B, N)[b][rows[b]]) and np.all(np.diff(p) > 0)
    flat = (np.arange(B)[:, None] * N + rows).reshape(-1)
    assert np.array_equal(out["cache_kc"], out["kc"][flat]) and np.array_equal(out["cache_vs"], out["vs"][flat])
    # K >= Nv keeps everything, K = 0 keeps text only
    full = oracle.prefill_layer(W, x, pos, B, N, 2, Nv, Nv + 7, cos, sin)
    assert full["n_keep"] == N and np.array_equal(full["pos_next"], pos)
    none = oracle.prefill_layer(W, x, pos, B, N, 2, Nv, 0, cos, sin)
    assert none["n_keep"] == shape.Nt and none["Nv_next"] == 0


# ---- decode over the pruned 4-bit KV cache --------------------------------------------------

def test_dequant_kv_equals_the_quantizers_own_xhat():
    x = (wl.rng(11, "kv").standard_normal((9, 256)) * 3).astype(np.float16)
    codes, scales, xhat = oracle.kv_quant(x)
    assert np.array_equal(oracle.dequant_kv(codes, scales), xhat)


def test_decode_attention_closed_forms():
    r = wl.rng(12, "dec")
    B, H, dh = 2, 3, 64
    q = r.standard_normal((B, H * dh)).astype(np.float16)
    k = r.standard_normal((B * 5, H * dh)).astype(np.float16)
    v = r.standard_normal((B * 5, H * dh)).astype(np.float16)
    kc, ks, _ = oracle.kv_quant(k)
    vc, vs, vhat = oracle.kv_quant(v)
    sh = lambda a: a.reshape(B, 5, -1)
    # a cache of one row: softmax over one key is 1, the output is that row's dequantized V
    o1 = oracle.decode_attention(q, sh(kc)[:, :1], sh(ks)[:, :1], sh(vc)[:, :1], sh(vs)[:, :1], H, dh)
    assert np.array_equal(o1, sh(vhat)[:, 0])
    # identical keys: uniform probabilities, the output is the mean of the dequantized V rows
    kc_same = np.repeat(sh(kc)[:, :1], 5, axis=1)
    ks_same = np.repeat(sh(ks)[:, :1], 5, axis=1)
    o2 = oracle.decode_attention(q, kc_same, ks_same, sh(vc), sh(vs), H, dh)
    mean = sh(vhat).astype(np.float64).mean(axis=1)
    assert np.allclose(o2.astype(np.float64), mean, rtol=0, atol=2e-3 * np.abs(mean).max())
    assert np.max(np.abs(o2.astype(np.float64) - mean)) <= np.max(np.spacing(np.abs(mean).astype(np.float16))).astype(np.float64)
    # a query of zeros gives uniform probabilities whatever the keys are
    o3 = oracle.decode_attention(np.zeros_like(q), sh(kc), sh(ks), sh(vc), sh(vs), H, dh)
    assert np.array_equal(o3, o2)


def test_decode_step_equals_last_row_of_a_longer_prefill():
    """Causality: with nothing pruned, the last token of an N-token prefill sees exactly what a decode
    step sees that follows an (N-1)-token prefill -- same K/V codes, same attention row, same output."""
    shape, W, x, pos, cos, sin = _small_layer(3)
    B, N, Nv, d = shape.B, shape.N, shape.Nv, 128
    full = oracle.prefill_layer(W, x, pos, B, N, 0, Nv, Nv, cos, sin)
    xb, pb = x.reshape(B, N, d), pos.reshape(B, N)
    head = oracle.prefill_layer(W, xb[:, :N - 1].reshape(-1, d), pb[:, :N - 1].reshape(-1), B, N - 1, 0, Nv, Nv,
                                cos, sin)
    cache = oracle.cache_from_prefill(head, B)
    assert cache["kc"].shape == (B, N - 1, d)
    dec = oracle.decode_layer(W, xb[:, N - 1], pb[:, N - 1], cache, cos, sin)
    last = np.arange(B) * N + N - 1
    assert np.array_equal(dec["kc"], full["kc"][last]) and np.array_equal(dec["vs"], full["vs"][last])
    assert np.array_equal(dec["cache"]["kc"].reshape(B * N, d), full["cache_kc"])
    for key in ("q", "o", "x1", "gu", "z", "x_next"):
        assert np.array_equal(dec[key], full[key][last]), key


def test_decode_reads_only_its_own_sequence_and_all_of_its_cache():
    shape, W, x, pos, cos, sin = _small_layer(4)
    B, N, Nv, d = shape.B, shape.N, shape.Nv, 128
    head = oracle.prefill_layer(W, x, pos, B, N, 0, Nv, 5, cos, sin)       # pruned cache: 5 visual + text
    cache = oracle.cache_from_prefill(head, B)
    xn = wl.rng(4, "new").standard_normal((B, d)).astype(np.float16)
    pn = np.full(B, N, np.int32)
    cos, sin = wl.rope_tables(64, N + 1)
    a = oracle.decode_layer(W, xn, pn, cache, cos, sin)
    assert a["cache"]["kc"].shape[1] == 5 + shape.Nt + 1
    # changing sequence 1's cache leaves sequence 0 untouched
    c2 = {k: v.copy() for k, v in cache.items()}
    c2["vc"][1] = -c2["vc"][1].clip(-7, 7)
    b = oracle.decode_layer(W, xn, pn, c2, cos, sin)
    assert np.array_equal(a["x_next"][0], b["x_next"][0]) and not np.array_equal(a["o"][1], b["o"][1])
    # dropping a cached row changes the output of that sequence (every row is read)
    c3 = {k: v[:, 1:] for k, v in cache.items()}
    c = oracle.decode_layer(W, xn, pn, c3, cos, sin)
    assert not np.array_equal(a["o"], c["o"])


# ---- offline budget allocation (Eq. 1-5) -----------------------------------------------------

def test_recipe_eq1_sensitivity_closed_forms():
    rec = oracle.recipe
    ref = np.array([2.0, 4.0, 8.0])
    assert rec.sensitivity(np.zeros(3), ref, 1e-6) == 0.0                       # x^q == x
    assert abs(rec.sensitivity(ref, ref, 0.0) - 1.0) < 1e-15                    # x^q == 0
    assert rec.sensitivity([1.0, 9.0, 2.0], [10.0, 10.0, 10.0], 0.0) == 0.2     # median, not mean
    assert rec.sensitivity([1.0, 3.0], [10.0, 10.0], 0.0) == pytest.approx(0.2)  # even count: mid-point
    a, b = wl.rng(1, "sens").uniform(0.1, 1, 9), wl.rng(2, "sens").uniform(1, 2, 9)
    assert rec.sensitivity(3 * a, 3 * b, 0.0) == pytest.approx(rec.sensitivity(a, b, 0.0), rel=1e-14)
    assert rec.sensitivity(a, b, 0.5) < rec.sensitivity(a, b, 0.0)              # eta only damps


def test_recipe_eq2_worked_example_and_library_percentile(golden_dir):
    rec = oracle.recipe
    rows = [l.split() for l in open(os.path.join(golden_dir, "recipe_eq2_worked.txt")) if l[0] != "#"]
    S = np.array([float(r[0]) for r in rows])
    want = np.array([float(r[1]) for r in rows])
    assert np.allclose(rec.normalize_sensitivity(S), want, rtol=0, atol=1e-15)
    x = wl.rng(3, "pct").uniform(0, 10, 11)
    for p in (10.0, 90.0, 37.5):
        assert rec.percentile_linear(x, p) == pytest.approx(np.percentile(x, p), rel=1e-14)
    # invariant to positive affine maps of the raw sensitivities; flat input -> 0.5
    assert np.allclose(rec.normalize_sensitivity(3 * x + 7), rec.normalize_sensitivity(x), atol=1e-13)
    assert np.array_equal(rec.normalize_sensitivity(np.full(4, 2.5)), np.full(4, 0.5))
    out = rec.normalize_sensitivity(x)
    assert out.min() == 0.1 and out.max() == 0.9                                 # heavy tails are capped


def test_recipe_eq3_shares():
    rec = oracle.recipe
    s = np.array([0.1, 0.5, 0.9, 0.3])
    pi = rec.layer_shares(s, 0.7)
    assert abs(pi.sum() - 1.0) < 1e-15 and np.all(pi > 0)
    assert np.array_equal(np.argsort(-pi), np.argsort(s))                        # less sensitive, larger drop share
    assert np.allclose(rec.layer_shares(np.full(5, 0.4), 0.3), 0.2)              # equal sensitivities: uniform
    assert np.allclose(rec.layer_shares(s, 1e9), 0.25, atol=1e-9)                # tau -> inf: uniform
    two = rec.layer_shares(np.array([0.2, 0.8]), 0.5)                            # m = 2 closed form: logistic
    assert two[0] == pytest.approx(1.0 / (1.0 + math.exp(-(0.8 - 0.2) / 0.5)), rel=1e-14)
    assert rec.layer_shares(s, 0.05).max() > 0.98                                # small tau: winner takes all


def test_recipe_eq4_eq5_schedule_and_budgets(golden_dir):
    rec = oracle.recipe
    m, p_min = 6, 0.3
    r = rec.keep_schedule(np.full(m, 1.0 / m), p_min)                            # uniform shares: a straight ramp
    assert np.allclose(r, 1.0 - (1.0 - p_min) * np.arange(1, m + 1) / m, atol=1e-15)
    pi = rec.layer_shares(rec.normalize_sensitivity(wl.rng(4, "S").uniform(0.01, 0.2, 9)), 1.0)
    r = rec.keep_schedule(pi, p_min)
    assert np.all(np.diff(r) <= 0) and r.min() >= p_min and r[0] < 1.0
    assert r[-1] == pytest.approx(p_min, abs=1e-15)                              # the whole drop budget is spent
    K = rec.budgets(r, 576)
    assert np.all(np.diff(K) <= 0) and K[-1] == 173                              # Table 4: 173 of 576 at ratio 0.3
    assert rec.budgets([1.0, 0.0, 0.25, 0.1], 580).tolist() == [580, 0, 145, 58]  # integers are not bumped
    full = rec.make_recipe(np.array([1.0, 2.0, 3.0, 4.0, 5.0]), 1.0, 0.3, 576)
    assert np.allclose(full["s_norm"], [0.1, 0.1875, 0.5, 0.8125, 0.9]) and full["K"][-1] == 173


def test_gflops_ratio_closed_forms():
    rec = oracle.recipe
    d, F, V0, T, L = 4096, 11008, 576, 64, 32
    assert rec.gflops_ratio([V0] * L, V0, T, d, F) == 100.0                      # nothing pruned
    # everything pruned in every layer: only the text tokens run
    assert rec.gflops_ratio([0] * L, V0, T, d, F) == pytest.approx(100.0 * rec.layer_cost(T, d, F) / rec.layer_cost(T + V0, d, F))
    # one layer of S tokens against the hand count 2 S (4 d^2 + 3 d F) + 4 S^2 d
    assert rec.layer_cost(10, 8, 16) == 2 * 10 * (4 * 64 + 3 * 8 * 16) + 4 * 100 * 8
    # pruning earlier saves more than pruning later with the same final count (the appendix's remark)
    early = [V0] * 2 + [173] * 30
    late = [V0] * 16 + [173] * 16
    assert rec.gflops_ratio(early, V0, T, d, F) < rec.gflops_ratio(late, V0, T, d, F) < 100.0
    # a constant vision-tower / projector term only pulls the ratio towards 100 %
    assert rec.gflops_ratio(early, V0, T, d, F, F_vt=1e12) > rec.gflops_ratio(early, V0, T, d, F)
    # the cost is dominated by the token-wise term at these lengths: ratio close to the token ratio
    r = rec.gflops_ratio(early, V0, T, d, F)
    tok = 100.0 * (2 * (V0 + T) + 30 * (173 + T)) / (32 * (V0 + T))
    assert abs(r - tok) < 1.5


# ---- grouped-query attention (the Qwen2.5-VL shape of the paper's second model) ---------------

def test_gqa_attention_equals_mha_with_replicated_kv_heads():
    """Grouped-query attention is multi-head attention in which every K/V head serves a group of
    query heads: replicating the K/V heads must give the already pinned multi-head result."""
    r = wl.rng(21, "gqa")
    B, N, H, Hkv, dh, vb, Nv = 2, 19, 6, 2, 64, 2, 11
    q = r.standard_normal((B * N, H * dh)).astype(np.float16)
    _, _, khat = oracle.kv_quant(r.standard_normal((B * N, Hkv * dh)).astype(np.float16))
    _, _, vhat = oracle.kv_quant(r.standard_normal((B * N, Hkv * dh)).astype(np.float16))
    o, ci, cv = oracle.attention(q, khat, vhat, B, N, H, dh, vb, Nv, Hkv=Hkv)
    rep = lambda a: np.repeat(a.reshape(B * N, Hkv, dh), H // Hkv, axis=1).reshape(B * N, H * dh)
    o2, ci2, cv2 = oracle.attention(q, rep(khat), rep(vhat), B, N, H, dh, vb, Nv)
    assert np.array_equal(o, o2) and np.array_equal(ci, ci2) and np.array_equal(cv, cv2)
    # and the decode read of the same rows
    kc, ks, _ = oracle.kv_quant(khat)
    vc, vs, _ = oracle.kv_quant(vhat)
    sh = lambda a: a.reshape(B, N, -1)
    d1 = oracle.decode_attention(q.reshape(B, N, -1)[:, -1], sh(kc), sh(ks), sh(vc), sh(vs), H, dh, Hkv)
    kc2, ks2, _ = oracle.kv_quant(rep(khat))
    vc2, vs2, _ = oracle.kv_quant(rep(vhat))
    d2 = oracle.decode_attention(q.reshape(B, N, -1)[:, -1], sh(kc2), sh(ks2), sh(vc2), sh(vs2), H, dh)
    assert np.array_equal(d1, d2)


def _small_gqa_layer(seed):
    shape = wl.Shape("g", d=256, H=4, F=160, layers=1, B=2, Nv=12, Nt=4, n_outlier=2, vis_begin=0)
    Hkv, dh, d = 2, 64, 256
    r = wl.rng(seed, "gqa-w")
    mk = lambda n, k: oracle.quantize_weights((r.standard_normal((n, k)) * 0.02).astype(np.float32))
    W = oracle.LayerWeights(qkv=mk(d + 2 * Hkv * dh, d), o=mk(d, d), gu=mk(2 * 160, d), down=mk(d, 160),
                            gamma1=np.ones(d, np.float32), gamma2=np.ones(d, np.float32), eps=1e-5,
                            H=4, dh=dh, F=160, Hkv=Hkv)
    x = wl.hidden_state(shape, seed)
    pos = wl.positions(shape)
    cos, sin = wl.rope_tables(dh, shape.N + 1)
    return shape, W, x, pos, cos, sin


def test_gqa_layer_cache_width_and_decode_consistency():
    shape, W, x, pos, cos, sin = _small_gqa_layer(6)
    B, N, Nv, d = shape.B, shape.N, shape.Nv, 256
    full = oracle.prefill_layer(W, x, pos, B, N, 0, Nv, Nv, cos, sin)
    assert full["cache_kc"].shape == (B * N, 128) and full["cache_ks"].shape == (B * N, 2)     # K/V heads only
    xb, pb = x.reshape(B, N, d), pos.reshape(B, N)
    head = oracle.prefill_layer(W, xb[:, :N - 1].reshape(-1, d), pb[:, :N - 1].reshape(-1), B, N - 1, 0, Nv, Nv,
                                cos, sin)
    dec = oracle.decode_layer(W, xb[:, N - 1], pb[:, N - 1], oracle.cache_from_prefill(head, B), cos, sin)
    last = np.arange(B) * N + N - 1
    for key in ("q", "o", "x1", "x_next"):
        assert np.array_equal(dec[key], full[key][last]), key
    assert np.array_equal(dec["kc"], full["kc"][last])


# ------------------------------------------------ block wiring of the layer composite
def _llama_block_fp64(x, Wqkv, Wo, Wgu, Wd, g1, g2, eps, H, dh, pos, mistake=None):
    """A LLaMA-style decoder block in plain fp64 numpy, written without the oracle: RMSNorm -> q|k|v
    projection -> rotate-half RoPE on q and k -> causal softmax attention -> output projection +
    residual -> RMSNorm -> gate|up projection -> SiLU(gate) * up -> down projection + residual.
    No quantizer anywhere.  `mistake` plants one wiring error (negative controls)."""
    N, d = x.shape
    F = Wd.shape[1]
    norm = lambda t, g: t / np.sqrt((t * t).mean(axis=1, keepdims=True) + eps) * g
    h = norm(x, g1)
    qkv = (x if mistake == "no_norm_before_qkv" else h) @ Wqkv.T
    q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    if mistake == "k_v_swapped":
        k, v = v, k
    inv = 1.0e4 ** (-np.arange(0, dh, 2) / dh)
    ang = pos[:, None] * inv[None, :]
    cos, sin = np.cos(ang), np.sin(ang)

    def rope(t):
        t = t.reshape(N, H, dh)
        a, b = t[..., :dh // 2], t[..., dh // 2:]
        return np.concatenate([a * cos[:, None] - b * sin[:, None], b * cos[:, None] + a * sin[:, None]], axis=-1).reshape(N, d)

    q = rope(q)
    if mistake != "k_not_rotated":
        k = rope(k)
    if mistake == "v_rotated":
        v = rope(v)
    o = np.zeros((N, d))
    for hd in range(H):
        sl = slice(hd * dh, (hd + 1) * dh)
        s = q[:, sl] @ k[:, sl].T / np.sqrt(dh)
        s = np.where(np.tril(np.ones((N, N), bool)), s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        o[:, sl] = (p / p.sum(axis=1, keepdims=True)) @ v[:, sl]
    x1 = (h if mistake == "residual_is_normed_input" else x) + o @ Wo.T
    h2 = norm(x1, g2)
    gu = h2 @ Wgu.T
    g, u = (gu[:, F:], gu[:, :F]) if mistake == "gate_up_swapped" else (gu[:, :F], gu[:, F:])
    z = g / (1.0 + np.exp(-g)) * u
    xn = (x if mistake == "second_residual_is_block_input" else x1) + z @ Wd.T
    return dict(attn_branch=x1 - x, ffn_branch=xn - x1, x1=x1, x_next=xn, q=q, k=k, v=v, o=o, gu=gu, z=z)


def test_layer_wiring_against_an_independent_fp64_block():
    """Pins WHICH tensor feeds which step in oracle/layer.py (residual sources, RMSNorm output into
    the projections, q|k|v and gate|up row order, what is rotated).  The reference is the plain fp64
    block above run on the dequantized W4 weights; the oracle adds int4 activation and 4-bit K/V
    noise (about 12 % of a GEMM output's rms each), so the two branch outputs must agree in
    direction (cosine > 0.85) and size (within 25 %), and so must the tensors between the steps (rotated
    q, the 4-bit K and V, attention output, gate|up, SwiGLU product); every planted wiring mistake drops
    the tensor or branch it touches below 0.75 or out of the size band.  Larger weights than the workload's make both branches
    comparable to the residual stream so that no term hides behind it."""
    d, H, dh, F, Nv, Nt = 256, 4, 64, 512, 40, 8
    N = Nv + Nt
    r = R(77)
    # rows of very different size and uneven gains: skipping a normalisation or using its output as the
    # residual changes sizes, not only directions
    x = (r.standard_normal((N, d)) * r.uniform(0.5, 4.0, (N, 1))).astype(np.float16)
    pos = (300 + 7 * np.arange(N)).astype(np.int32)       # non-contiguous position ids, as after pruning
    g1 = r.uniform(0.3, 2.0, d).astype(np.float32)
    g2 = r.uniform(0.3, 2.0, d).astype(np.float32)
    fw = dict(qkv=r.standard_normal((3 * d, d)) * 0.08, o=r.standard_normal((d, d)) * 0.08,
              gu=r.standard_normal((2 * F, d)) * 0.08, down=r.standard_normal((d, F)) * 0.08)
    q = {k_: oracle.quantize_weights(v_.astype(np.float32)) for k_, v_ in fw.items()}
    deq = {k_: c.astype(np.float64) * np.repeat(s_.astype(np.float64), 128, axis=1)[:, :c.shape[1]] for k_, (c, s_) in q.items()}
    W = oracle.LayerWeights(qkv=q["qkv"], o=q["o"], gu=q["gu"], down=q["down"], gamma1=g1, gamma2=g2, eps=1e-5,
                            H=H, dh=dh, F=F)
    cos, sin = wl.rope_tables(dh, int(pos.max()) + 1)
    out = oracle.prefill_layer(W, x, pos, 1, N, 0, Nv, Nv, cos, sin)           # K = Nv: nothing pruned
    xf = x.astype(np.float64)
    got = dict(attn_branch=out["x1"].astype(np.float64) - xf, ffn_branch=out["x_next"].astype(np.float64) - out["x1"].astype(np.float64))
    for name, key in dict(q="q", k="khat", v="vhat", o="o", gu="gu", z="z").items():      # tensors between the steps
        got[name] = out[key].astype(np.float64)

    def agree(a, b):
        a, b = a.ravel(), b.ravel()
        return float(a @ b / np.sqrt((a @ a) * (b @ b))), float(np.sqrt((a @ a) / (b @ b)))

    ref = _llama_block_fp64(xf, deq["qkv"], deq["o"], deq["gu"], deq["down"], g1, g2, 1e-5, H, dh, pos.astype(np.float64))
    for branch in ("q", "k", "v", "o", "gu", "z", "attn_branch", "ffn_branch"):
        c, ratio = agree(got[branch], ref[branch])
        print(branch, round(c, 3), round(ratio, 3))
        assert c > 0.85 and 0.75 < ratio < 1.25, (branch, c, ratio)
    for branch in ("attn_branch", "ffn_branch"):
        # the branch is not hidden behind the residual stream
        assert np.sqrt((ref[branch] ** 2).mean()) > 0.2 * np.sqrt((xf ** 2).mean())
    # negative controls: each planted mistake must break the agreement of the branch it touches
    touched = dict(no_norm_before_qkv="q", k_v_swapped="k", k_not_rotated="k", v_rotated="v",
                   residual_is_normed_input="attn_branch", gate_up_swapped="z")
    for mistake, branch in touched.items():
        bad = _llama_block_fp64(xf, deq["qkv"], deq["o"], deq["gu"], deq["down"], g1, g2, 1e-5, H, dh,
                                pos.astype(np.float64), mistake=mistake)
        c, ratio = agree(got[branch], bad[branch])
        print(mistake, round(c, 3), round(ratio, 3))
        assert c < 0.75 or not 0.75 < ratio < 1.25, (mistake, c, ratio)

    # The two residual sources, exactly: what a projection adds is the fp64 product of ITS dequantized
    # operands, so (block output - that product) must be the residual tensor up to the fp16 rounding
    # of the sum -- and must not be any other tensor of the block.
    def deq_act(qa, sa):
        return qa.astype(np.float64) * sa.astype(np.float64)[:, None]

    add_o = deq_act(out["qa2"], out["sa2"]) @ deq["o"].T
    add_d = deq_act(out["qa4"], out["sa4"]) @ deq["down"].T
    x1f, xnf = out["x1"].astype(np.float64), out["x_next"].astype(np.float64)
    tol = lambda t: 2.0 ** -10 * np.maximum(np.abs(t), 1.0)
    assert np.all(np.abs((x1f - add_o) - xf) <= tol(x1f))                    # first residual: the block input
    assert np.all(np.abs((xnf - add_d) - x1f) <= tol(xnf))                   # second residual: x1
    assert not np.all(np.abs((x1f - add_o) - out["h1"].astype(np.float64)) <= tol(x1f))
    assert not np.all(np.abs((xnf - add_d) - xf) <= tol(xnf))
    assert not np.all(np.abs((xnf - add_d) - out["h2"].astype(np.float64)) <= tol(xnf))


# ------------------------------------------------ sensitivity profiling (Eq. 1 inputs)
def _profiler_case(seed, B=2, d=128, H=4, Hkv=2, dh=32, F=192, N=24, scale=0.08):
    from oracle import profiler
    r = R(seed)
    x = (r.standard_normal((B * N, d)) * r.uniform(0.5, 3.0, (B * N, 1))).astype(np.float16)
    pos = np.tile(5 + 3 * np.arange(N), B).astype(np.int32)
    dq = (H + 2 * Hkv) * dh
    W = profiler.FullPrecisionWeights(
        qkv=(r.standard_normal((dq, d)) * scale).astype(np.float16), o=(r.standard_normal((d, d)) * scale).astype(np.float16),
        gu=(r.standard_normal((2 * F, d)) * scale).astype(np.float16), down=(r.standard_normal((d, F)) * scale).astype(np.float16),
        gamma1=r.uniform(0.5, 1.5, d).astype(np.float32), gamma2=r.uniform(0.5, 1.5, d).astype(np.float32),
        eps=1e-5, H=H, dh=dh, F=F, Hkv=Hkv)
    cos, sin = wl.rope_tables(dh, int(pos.max()) + 100)
    return profiler, W, x, pos, B, N, cos, sin


def test_full_precision_block_against_torch_library_ops():
    """The quantizer-free block of the profiler, rebuilt from torch's own routines (rms_norm, linear,
    scaled_dot_product_attention with is_causal and grouped heads, silu) in fp64; RoPE has no library
    routine and is pinned by the tests below, so here every position id is 0 (the identity rotation)."""
    profiler, W, x, pos, B, N, cos, sin = _profiler_case(3)
    F_ = torch.nn.functional
    got = profiler.block_full_precision(W, x, np.zeros_like(pos), B, N, cos, sin)
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    d, H, Hkv, dh = W.H * W.dh, W.H, W.Hkv, W.dh
    xt = t(x).reshape(B, N, d)
    qkv = F_.linear(F_.rms_norm(xt, (d,), t(W.gamma1), W.eps), t(W.qkv))
    q = qkv[..., :d].reshape(B, N, H, dh).transpose(1, 2)
    k = qkv[..., d:d + Hkv * dh].reshape(B, N, Hkv, dh).transpose(1, 2)
    v = qkv[..., d + Hkv * dh:].reshape(B, N, Hkv, dh).transpose(1, 2)
    o = F_.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True).transpose(1, 2).reshape(B, N, d)
    x1 = xt + F_.linear(o, t(W.o))
    gu = F_.linear(F_.rms_norm(x1, (d,), t(W.gamma2), W.eps), t(W.gu))
    want = x1 + F_.linear(F_.silu(gu[..., :W.F]) * gu[..., W.F:], t(W.down))
    assert np.allclose(got, want.reshape(B * N, d).numpy(), rtol=1e-10, atol=1e-10)
    # grouped heads matter in this case: reading K/V head h instead of h // (H/Hkv) would differ
    assert W.H != W.Hkv


def test_full_precision_block_rope_and_masking_properties():
    """What fixes the rotation and the mask inside the block: attention sees only position
    DIFFERENCES (shifting every id by a constant changes nothing, stretching them does), a token
    never sees a later one, and the samples of a batch do not mix."""
    profiler, W, x, pos, B, N, cos, sin = _profiler_case(4)
    base = profiler.block_full_precision(W, x, pos, B, N, cos, sin)
    shifted = profiler.block_full_precision(W, x, pos + 17, B, N, cos, sin)
    assert np.allclose(base, shifted, rtol=0, atol=2e-5)   # the cos/sin tables are fp32
    stretched = profiler.block_full_precision(W, x, (pos - 5) * 2, B, N, cos, sin)
    assert np.abs(base - stretched).max() > 1e-3
    # the rotation acts on q and k only: with every id 0 and one token per sequence the block is
    # position-free, with two tokens the second one's output depends on its distance to the first
    x2 = x.copy()
    x2[N - 1] += 1.0                                    # last token of sample 0
    pert = profiler.block_full_precision(W, x2, pos, B, N, cos, sin)
    assert np.array_equal(pert[:N - 1], base[:N - 1])   # causal: earlier tokens unchanged
    assert np.abs(pert[N - 1] - base[N - 1]).max() > 1e-2
    assert np.array_equal(pert[N:], base[N:])           # the other sample unchanged
    x3 = x.copy()
    x3[0] += 1.0                                        # first token: every later one of its sample moves
    pert = profiler.block_full_precision(W, x3, pos, B, N, cos, sin).reshape(B, N, -1)
    assert np.all(np.abs(pert[0] - base.reshape(B, N, -1)[0]).max(axis=1) > 1e-6)


def test_full_precision_block_rotation_against_complex_multiplication():
    """Rotate-half RoPE is multiplication of (x_i + j x_{i+dh/2}) by exp(j pos theta_i): a single
    head, single token block cannot show it (softmax over one key), so check the q.k logits the
    block must produce through a 2-token sequence whose value vectors make the output read off the
    attention weight."""
    from oracle import profiler
    r = R(9)
    dh, P = 32, 64
    cos, sin = wl.rope_tables(dh, P)
    t = r.standard_normal((3, dh))
    pos = np.array([3, 11, 40])
    got = profiler._rotate(t.copy(), 1, dh, cos[pos].astype(np.float64), sin[pos].astype(np.float64))
    inv = 1.0e4 ** (-np.arange(0, dh, 2) / dh)
    z = (t[:, :dh // 2] + 1j * t[:, dh // 2:]) * np.exp(1j * pos[:, None] * inv[None, :])
    want = np.concatenate([z.real, z.imag], axis=1)
    assert np.allclose(got, want, rtol=0, atol=1e-6)    # the tables are fp32


def test_full_precision_block_closed_forms():
    """Zero projections: with W_o = 0 and W_down = 0 the block is the identity (both residuals start
    from the right tensor); with only W_down = 0 the output is x + o W_o^T, and a constant value
    projection makes o that constant whatever the attention weights are."""
    profiler, W, x, pos, B, N, cos, sin = _profiler_case(5)
    import dataclasses
    xf = x.astype(np.float64)
    Z = dataclasses.replace(W, o=np.zeros_like(W.o), down=np.zeros_like(W.down))
    assert np.array_equal(profiler.block_full_precision(Z, x, pos, B, N, cos, sin), xf)
    # v rows of the qkv weight chosen so that v = c for every token: needs h @ Wv^T = c; use one
    # token per sequence (N = 1), where attention is the identity on v whatever q and k are
    one = dataclasses.replace(W, down=np.zeros_like(W.down))
    got = profiler.block_full_precision(one, x[:B], pos[:B], B, 1, cos, sin)
    d, dkv = W.H * W.dh, W.Hkv * W.dh
    g1 = W.gamma1.astype(np.float64)
    h = xf[:B] / np.sqrt((xf[:B] ** 2).mean(axis=1, keepdims=True) + W.eps) * g1
    v = h @ W.qkv.astype(np.float64)[d + dkv:].T                         # [B, dkv]
    o = np.repeat(v.reshape(B, W.Hkv, W.dh), W.H // W.Hkv, axis=1).reshape(B, d)
    assert np.allclose(got, xf[:B] + o @ W.o.astype(np.float64).T, rtol=1e-12, atol=1e-12)


def test_activation_deviation_and_profile():
    """Eq. 1's two norms against numpy's norm, per sample; and the profile itself: identical runs
    give S = 0, the low-bit run of the pinned layer composite against the full-precision block
    gives a deviation of int4 size, and putting the weights on their int4 grid (so that only the
    activation and K/V quantizers remain) lowers it."""
    profiler, W, x, pos, B, N, cos, sin = _profiler_case(6, B=3)
    r = R(10)
    a, b = r.standard_normal((B * N, 16)), r.standard_normal((B * N, 16))
    dn, rn = profiler.activation_deviation(a, b, B)
    for i in range(B):
        sl = slice(i * N, (i + 1) * N)
        assert math.isclose(dn[i], np.linalg.norm((a - b)[sl]), rel_tol=1e-12)
        assert math.isclose(rn[i], np.linalg.norm(b[sl]), rel_tol=1e-12)
    dn, rn = profiler.activation_deviation(b, b, B)
    assert np.all(dn == 0) and oracle.recipe.sensitivity(dn, rn, 1e-6) == 0.0
    dn, _ = profiler.activation_deviation(3.0 * b, b, B)                  # x^q = 3x: ratio exactly 2
    assert np.allclose(dn / rn, 2.0, rtol=1e-12)

    def quantized(Wf):
        q = {k_: oracle.quantize_weights(np.asarray(getattr(Wf, k_), np.float32)) for k_ in ("qkv", "o", "gu", "down")}
        return oracle.LayerWeights(qkv=q["qkv"], o=q["o"], gu=q["gu"], down=q["down"], gamma1=Wf.gamma1,
                                   gamma2=Wf.gamma2, eps=Wf.eps, H=Wf.H, dh=Wf.dh, F=Wf.F, Hkv=Wf.Hkv), q

    Wq, q = quantized(W)
    S_full = profiler.profile_sensitivity(Wq, W, x, pos, B, N, 0, N - 4, cos, sin)
    import dataclasses
    deq = {k_: (c.astype(np.float64) * np.repeat(s_.astype(np.float64), 128, axis=1)[:, :c.shape[1]]) for k_, (c, s_) in q.items()}
    on_grid = dataclasses.replace(W, **deq)
    S_act = profiler.profile_sensitivity(Wq, on_grid, x, pos, B, N, 0, N - 4, cos, sin)
    print("S with fp weights", S_full, " S with weights on the int4 grid", S_act)
    assert 0.0 < S_act < S_full < 0.5
    # the same number from its parts
    low = oracle.prefill_layer(Wq, x, pos, B, N, 0, N - 4, N - 4, cos, sin)["x_next"].astype(np.float64)
    full = profiler.block_full_precision(W, x, pos, B, N, cos, sin)
    ratios = [np.linalg.norm(low[i * N:(i + 1) * N] - full[i * N:(i + 1) * N]) / (np.linalg.norm(full[i * N:(i + 1) * N]) + 1e-6)
              for i in range(B)]
    assert math.isclose(S_full, float(np.median(ratios)), rel_tol=1e-12)
