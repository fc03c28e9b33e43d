"""GPU parity, per operation, through the C ABI: the HIP path against the CPU
oracle on identical seeded inputs.  Integer outputs (int4 codes, int32
accumulators, index sets, KV codes, fp16 scales) must be bit-exact; fp16
tensors must be within 1e-2 relative (|a-b| <= 1e-2 * max(|b|, rms(b))) and
fp32 scores within 1e-5 relative."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_17320_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def unpack4(p):
    """uint8 [..., n/2] nibble-packed (element 2j in the low nibble) -> int8 [..., n]."""
    p = np.asarray(p, np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), np.int16)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = p >> 4
    return ((out ^ 8) - 8).astype(np.int8)


def close_f16(a, b, tol=1e-2):
    a = a.astype(np.float64)
    b = b.astype(np.float64)
    rms = np.sqrt((b ** 2).mean()) if b.size else 0.0
    return np.all(np.abs(a - b) <= tol * np.maximum(np.abs(b), rms))


# ---------------------------------------------------------------- weights
@pytest.mark.parametrize("N,K", [(64, 1376), (128, 512), (192, 4096)])
def test_quantize_and_pack_weights(qb, N, K):
    from paper_2604_17320_amd.model import PackedLinear
    w = (wl.rng(3, "w", N, K).standard_normal((N, K), dtype=np.float32) * np.float32(0.02))
    w[1, :128] = 0
    codes, scales = oracle.quantize_weights(w)
    lin = PackedLinear.from_fp32(dev(w), keep_plain=True)
    assert np.array_equal(host(lin.codes), codes)
    assert np.array_equal(host(lin.plain_scales).view(np.uint16), scales.view(np.uint16))
    # packed layout: [group][row][64 bytes], zero padded; scales [group][row]
    G = (K + 127) // 128
    pk = unpack4(host(lin.packed).reshape(G, N, 64))
    full = np.zeros((N, G * 128), np.int8)
    full[:, :K] = codes
    assert np.array_equal(pk, full.reshape(N, G, 128).transpose(1, 0, 2))
    assert np.array_equal(host(lin.scales).reshape(G, N).view(np.uint16), scales.T.view(np.uint16))


def test_pack_weights_rejects_bad_shapes(qb):
    W = qb.Weights(48, 512, 1, 1)
    z = torch.zeros(8, dtype=torch.int8, device="cuda")
    s = torch.zeros(8, dtype=torch.float16, device="cuda")
    with pytest.raises(qb.QuotaError) as e:
        qb.quota_pack_weights(z, s, W)
    assert e.value.code == qb.ERR_SHAPE
    W = qb.Weights(64, 500, 1, 1)
    with pytest.raises(qb.QuotaError):
        qb.quota_pack_weights(z, s, W)


# ------------------------------------------------------------ quantizers
def _act(M, d, seed, scale=1.0):
    x = wl.rng(seed, "act", M, d).standard_normal((M, d), dtype=np.float32) * np.float32(scale)
    x[:, :: max(1, d // 7)] *= 20
    return x.astype(np.float16)


@pytest.mark.parametrize("M,d", [(80, 512), (37, 1376), (640, 4096), (5, 11008), (3, 16384), (1, 8), (5, 18944), (2, 32768)])
def test_quantize_act_bit_exact(qb, M, d):
    x = _act(M, d, 11)
    if M > 2:
        x[2] = 0
    q, s, ss, rs = oracle.quantize_act(x)
    xd = dev(x)
    qp = torch.empty((M, d // 2), dtype=torch.uint8, device="cuda")
    sc = torch.empty(M, dtype=torch.float32, device="cuda")
    sq = torch.empty(M, dtype=torch.float32, device="cuda")
    rq = torch.empty(M, dtype=torch.float32, device="cuda")
    qb.quota_quantize_act(xd, M, d, d, qp, sc, sq, rq)
    assert np.array_equal(unpack4(host(qp)), q)
    assert np.array_equal(host(sc), s)
    assert np.array_equal(host(sq), ss) and np.array_equal(host(rq), rs)
    # without the side outputs (other kernel instantiation), and with a row stride
    qp2 = torch.zeros_like(qp)
    sc2 = torch.zeros_like(sc)
    if d % 16 == 0:
        qb.quota_quantize_act(xd, M, d // 2, d, qp2, sc2)
        q2, s2, _, _ = oracle.quantize_act(x[:, : d // 2])
        assert np.array_equal(unpack4(host(qp2).reshape(-1)[: M * d // 4].reshape(M, d // 4)), q2)
        assert np.array_equal(host(sc2), s2)


def test_quantize_act_errors(qb):
    x = torch.zeros((4, 64), dtype=torch.float16, device="cuda")
    q = torch.zeros((4, 32), dtype=torch.uint8, device="cuda")
    s = torch.zeros(4, dtype=torch.float32, device="cuda")
    for args, code in [((x, 4, 60, 64, q, s), qb.ERR_SHAPE), ((x, 4, 64, 32, q, s), qb.ERR_SHAPE),
                       ((x, -1, 64, 64, q, s), qb.ERR_INVALID_ARG), ((None, 4, 64, 64, q, s), qb.ERR_NULL),
                       ((x, 4, 32776, 32776, q, s), qb.ERR_SHAPE)]:
        with pytest.raises(qb.QuotaError) as e:
            qb.quota_quantize_act(*args)
        assert e.value.code == code
    qb.quota_quantize_act(x, 0, 64, 64, q, s)          # empty input is fine


@pytest.mark.parametrize("M,d", [(80, 512), (33, 4096), (6, 5120), (3, 18944)])
def test_rmsnorm_quantize_act(qb, M, d):
    x = _act(M, d, 12, 1.7)
    gamma = wl.rng(12, "gamma", d).uniform(0.5, 1.5, d).astype(np.float32)
    h = oracle.rmsnorm(x, gamma, 1e-5)
    q, s, _, _ = oracle.quantize_act(h)
    _, _, ss, rs = oracle.quantize_act(x)
    qp = torch.empty((M, d // 2), dtype=torch.uint8, device="cuda")
    sc, sq, rq = (torch.empty(M, dtype=torch.float32, device="cuda") for _ in range(3))
    hh = torch.empty((M, d), dtype=torch.float16, device="cuda")
    qb.quota_rmsnorm_quantize_act(dev(x), M, d, d, dev(gamma), 1e-5, qp, sc, sq, rq, hh)
    assert np.array_equal(host(hh).view(np.uint16), h.view(np.uint16))
    assert np.array_equal(unpack4(host(qp)), q) and np.array_equal(host(sc), s)
    assert np.array_equal(host(sq), ss) and np.array_equal(host(rq), rs)
    qp2 = torch.empty_like(qp)
    sc2 = torch.empty_like(sc)
    qb.quota_rmsnorm_quantize_act(dev(x), M, d, d, dev(gamma), 1e-5, qp2, sc2)
    assert torch.equal(qp2, qp) and torch.equal(sc2, sc)


@pytest.mark.parametrize("M,F", [(35, 1376), (9, 11008), (7, 18944), (2, 32768)])
def test_silu_mul_quantize_act(qb, M, F):
    gu = (_act(M, 2 * F, 13, 1.5))
    z = oracle.silu_mul(gu, F)
    q, s, _, _ = oracle.quantize_act(z)
    qp = torch.empty((M, F // 2), dtype=torch.uint8, device="cuda")
    sc = torch.empty(M, dtype=torch.float32, device="cuda")
    zz = torch.empty((M, F), dtype=torch.float16, device="cuda")
    qb.quota_silu_mul_quantize_act(dev(gu), M, F, qp, sc, zz)
    zg = host(zz)
    assert close_f16(zg, z)
    assert (zg.view(np.uint16) != z.view(np.uint16)).mean() < 5e-3      # fp32 vs fp64 silu
    # teacher-forced: with the oracle's z injected the codes are bit-exact
    qb.quota_silu_mul_quantize_act(dev(gu), M, F, qp, sc, None, dev(z))
    assert np.array_equal(unpack4(host(qp)), q) and np.array_equal(host(sc), s)


# ------------------------------------------------------------------ GEMM
def _gemm_case(M, N, K, seed):
    r = wl.rng(seed, "gemm", M, N, K)
    w = r.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    qw, sw = oracle.quantize_weights(w)
    x = _act(M, K, seed + 1)
    qa, sa, _, _ = oracle.quantize_act(x)
    res = r.standard_normal((M, N), dtype=np.float32).astype(np.float16)
    return qa, sa, qw, sw, res


def _pack4(codes):
    c = codes.astype(np.uint8) & 0xF
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


@pytest.mark.parametrize("M,N,K", [(80, 1536, 512), (35, 512, 1376), (300, 2752, 512), (129, 4096, 4096),
                                   (1, 64, 32), (640, 1536, 1376), (257, 320, 11008),
                                   (16, 4096, 4096), (7, 512, 1376), (16, 9216, 512), (13, 128, 11008)])
def test_w4a4_gemm_bit_exact(qb, M, N, K):
    from paper_2604_17320_amd.model import PackedLinear
    qa, sa, qw, sw, res = _gemm_case(M, N, K, 21)
    y_ref, acc_ref = oracle.w4a4_gemm(qa, sa, qw, sw, want_acc=True)
    yr_ref = oracle.w4a4_gemm(qa, sa, qw, sw, residual=res)
    lin = PackedLinear.from_codes(dev(qw), dev(sw))
    qad, sad = dev(_pack4(qa)), dev(sa)
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    qb.quota_w4a4_gemm(qad, sad, M, lin.desc, y, N)                     # fast kernel
    assert np.array_equal(host(y).view(np.uint16), y_ref.view(np.uint16))
    y2 = torch.empty((M, N + 8), dtype=torch.float16, device="cuda")
    qb.quota_w4a4_gemm(qad, sad, M, lin.desc, y2, N + 8, dev(res), N, acc)   # residual + int32 debug
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(host(y2)[:, :N].view(np.uint16), yr_ref.view(np.uint16))
    y3 = torch.empty((M, N), dtype=torch.float16, device="cuda")
    qb.quota_w4a4_gemm(qad, sad, M, lin.desc, y3, N, dev(res), N)
    assert np.array_equal(host(y3).view(np.uint16), yr_ref.view(np.uint16))


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
def test_w4a4_gemm_every_tile_bit_exact(qb, tile, pinned_gemm):
    """Each of the five tile instantiations, pinned with quota_set_gemm_variant, on shapes with ragged
    rows, a ragged last group and several column tiles."""
    from paper_2604_17320_amd.model import PackedLinear
    pinned_gemm(tile)
    for M, N, K in [(150, 1024, 1376), (70, 512, 4096)]:
        qa, sa, qw, sw, res = _gemm_case(M, N, K, 23)
        y_ref = oracle.w4a4_gemm(qa, sa, qw, sw, residual=res)
        lin = PackedLinear.from_codes(dev(qw), dev(sw))
        y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        qb.quota_w4a4_gemm(dev(_pack4(qa)), dev(sa), M, lin.desc, y, N, dev(res), N)
        assert np.array_equal(host(y).view(np.uint16), y_ref.view(np.uint16)), (tile, M, N, K)


def test_w4a4_gemm_unit_scales_give_exact_integers(qb):
    from paper_2604_17320_amd.model import PackedLinear
    r = wl.rng(5, "unit")
    M, N, K = 70, 128, 256
    qa = r.integers(-8, 8, (M, K)).astype(np.int8)
    qw = r.integers(-8, 8, (N, K)).astype(np.int8)
    lin = PackedLinear.from_codes(dev(qw), dev(np.ones((N, 2), np.float16)))
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    qb.quota_w4a4_gemm(dev(_pack4(qa)), dev(np.ones(M, np.float32)), M, lin.desc, y, N)
    exact = qa.astype(np.int64) @ qw.astype(np.int64).T       # |sum| <= 16384: one fp16 rounding
    assert np.array_equal(host(y), exact.astype(np.float16))


# -------------------------------------------------------- RoPE + KV quant
@pytest.mark.parametrize("H,dh,M", [(8, 64, 80), (32, 128, 70), (3, 128, 5)])
def test_rope_kv_quant_bit_exact(qb, H, dh, M):
    d = H * dh
    qkv = _act(M, 3 * d, 31, 2.0)
    qkv[3, d:d + 64] = 0
    n_pos = 700
    pos = wl.rng(31, "pos").integers(0, n_pos, M).astype(np.int32)
    cos, sin = wl.rope_tables(dh, n_pos)
    q_ref = oracle.rope(qkv[:, :d], H, dh, pos, cos, sin)
    k_ref = oracle.rope(qkv[:, d:2 * d], H, dh, pos, cos, sin)
    kc, ks, khat = oracle.kv_quant(k_ref)
    vc, vs, vhat = oracle.kv_quant(np.ascontiguousarray(qkv[:, 2 * d:]))
    f16 = lambda *s: torch.empty(s, dtype=torch.float16, device="cuda")
    u8 = lambda *s: torch.empty(s, dtype=torch.uint8, device="cuda")
    q_rot, kh, vh = f16(M, d), f16(M, d), f16(M, d)
    kcd, vcd, ksd, vsd = u8(M, d // 2), u8(M, d // 2), f16(M, d // 64), f16(M, d // 64)
    qb.quota_rope_kv_quant(dev(qkv), M, H, dh, dev(pos), dev(cos), dev(sin), n_pos, q_rot, kh, vh,
                           kcd, ksd, vcd, vsd)
    assert np.array_equal(host(q_rot).view(np.uint16), q_ref.view(np.uint16))
    assert np.array_equal(unpack4(host(kcd)), kc) and np.array_equal(unpack4(host(vcd)), vc)
    assert np.array_equal(host(ksd).view(np.uint16), ks.view(np.uint16))
    assert np.array_equal(host(vsd).view(np.uint16), vs.view(np.uint16))
    assert np.array_equal(host(kh).view(np.uint16), khat.view(np.uint16))
    assert np.array_equal(host(vh).view(np.uint16), vhat.view(np.uint16))


def test_kv_quant_append(qb):
    from paper_2604_17320_amd.model import KVCache4
    B, N, H, dh = 2, 24, 4, 128
    d = H * dh
    k = _act(B * N, d, 41, 2.0)
    v = _act(B * N, d, 42, 0.7)
    kc, ks, _ = oracle.kv_quant(k)
    vc, vs, _ = oracle.kv_quant(v)
    cache = KVCache4(B, 20, H, dh)
    rows = np.stack([np.sort(wl.rng(41, "rows", b).permutation(N)[:7]) for b in range(B)]).astype(np.int32)
    qb.quota_kv_quant_append(dev(k), dev(v), B, N, H, dh, None, 5, cache.desc)      # rows 0..4
    qb.quota_kv_quant_append(dev(k), dev(v), B, N, H, dh, dev(rows), 7, cache.desc)
    assert cache.len == 12
    for b in range(B):
        src = np.concatenate([np.arange(5), rows[b]]) + b * N
        assert np.array_equal(unpack4(host(cache.k_codes)[b, :12]), kc[src])
        assert np.array_equal(unpack4(host(cache.v_codes)[b, :12]), vc[src])
        assert np.array_equal(host(cache.k_scales)[b, :12].view(np.uint16), ks[src].view(np.uint16))
        assert np.array_equal(host(cache.v_scales)[b, :12].view(np.uint16), vs[src].view(np.uint16))
    with pytest.raises(qb.QuotaError) as e:
        qb.quota_kv_quant_append(dev(k), dev(v), B, N, H, dh, None, 9, cache.desc)
    assert e.value.code == qb.ERR_CAPACITY and cache.len == 12
    qb.quota_kv_quant_append(dev(k), dev(v), B, N, H, dh, None, 0, cache.desc)
    assert cache.len == 12


# ------------------------------------------------------------- attention
@pytest.mark.parametrize("B,N,H,dh,vb,Nv", [(1, 80, 8, 64, 0, 64), (2, 200, 3, 128, 5, 150),
                                             (1, 640, 4, 128, 0, 576), (1, 33, 2, 128, 0, 0)])
def test_attention_prefill_and_column_masses(qb, B, N, H, dh, vb, Nv):
    d = H * dh
    q = _act(B * N, d, 51, 1.0)
    _, _, khat = oracle.kv_quant(_act(B * N, d, 52, 1.0))
    _, _, vhat = oracle.kv_quant(_act(B * N, d, 53, 1.0))
    o_ref, ci_ref, cv_ref = oracle.attention(q, khat, vhat, B, N, H, dh, vb, Nv)
    o = torch.empty((B * N, d), dtype=torch.float16, device="cuda")
    ci = torch.zeros((B, max(Nv, 1)), dtype=torch.float32, device="cuda")
    cv = torch.zeros((B, max(Nv, 1)), dtype=torch.float32, device="cuda")
    ws = torch.empty(qb.quota_attention_workspace_bytes(B, N, H, dh), dtype=torch.uint8, device="cuda")
    qb.quota_attention_prefill(dev(q), dev(khat), dev(vhat), B, N, H, dh, vb, Nv, o, ci, cv, ws)
    assert close_f16(host(o), o_ref)
    if Nv:
        cig, cvg = host(ci)[:, :Nv], host(cv)[:, :Nv]
        assert np.allclose(cig, ci_ref, rtol=2e-5, atol=1e-7), np.abs(cig / ci_ref - 1).max()
        assert np.allclose(cvg, cv_ref, rtol=2e-5, atol=1e-7), np.abs(cvg / cv_ref - 1).max()


# -------------------------------------------------------- score and top-k
def _metrics(B, Nv, seed):
    r = wl.rng(seed, "metrics", B, Nv)
    return (r.uniform(100, 9000, (B, Nv)).astype(np.float32), r.uniform(1, 400, (B, Nv)).astype(np.float32),
            r.uniform(0, 0.2, (B, Nv)).astype(np.float32), r.uniform(0, 3, (B, Nv)).astype(np.float32))


@pytest.mark.parametrize("B,Nv", [(1, 64), (3, 576), (2, 2880), (1, 1), (1, 3072), (2, 7), (2, 4100), (1, 8192)])
def test_score_tokens_bit_exact(qb, B, Nv):
    ss, rs, ci, cv = _metrics(B, Nv, 61)
    if Nv > 4:
        cv[0] = 0.25                                    # a flat metric -> 0.5
        ci[0, :3] = ci[0, 3]                            # ties among the order statistics
    for kw in [dict(), dict(w_m=0.0, w_c=0.5333, w_s=0.1833, w_r=0.2833), dict(p_lo=0, p_hi=100),
               dict(p_lo=25, p_hi=50)]:
        sc_ref, g_ref = oracle.score(ss, rs, ci, cv, want_normed=True, **kw)
        p = qb.quota_score_params_default()
        for k, v in kw.items():
            setattr(p, {"p_lo": "pct_lo", "p_hi": "pct_hi"}.get(k, k), v)
        sc = torch.empty((B, Nv), dtype=torch.float32, device="cuda")
        g = torch.empty((4, B, Nv), dtype=torch.float32, device="cuda")
        qb.quota_score_tokens(dev(ss), dev(rs), dev(ci), dev(cv), B, Nv, p, sc, g)
        assert np.array_equal(host(g), g_ref)
        assert np.array_equal(host(sc), sc_ref)


def test_score_tokens_from_hidden(qb):
    shape = wl.CONFIGS[0]
    x = wl.hidden_state(shape, 7)
    B, N, Nv, d = 1, shape.N, shape.Nv, shape.d
    _, _, ss, rs = oracle.quantize_act(x[:Nv])
    _, _, ci, cv = _metrics(B, Nv, 62)
    sc_ref = oracle.score(ss[None], rs[None], ci, cv)
    sc = torch.empty((B, Nv), dtype=torch.float32, device="cuda")
    ws = torch.empty(2 * B * Nv, dtype=torch.float32, device="cuda")
    qb.quota_score_tokens_from_hidden(dev(x), B, Nv, d, d, N * d, dev(ci), dev(cv),
                                      qb.quota_score_params_default(), sc, None, ws)
    assert np.array_equal(host(sc), sc_ref)


@pytest.mark.parametrize("B,Nv", [(1, 64), (3, 576), (2, 2880), (1, 3072), (2, 5), (2, 4100), (1, 8192)])
def test_topk_prune_bit_exact(qb, B, Nv):
    r = wl.rng(71, "topk", B, Nv)
    sc = (np.round(r.uniform(0, 1, (B, Nv)) * 50) / 50).astype(np.float32)     # plenty of ties
    if Nv > 10:
        sc[0, 5] = np.nan
        sc[0, 7] = -0.0
        sc[0, 8] = 0.0
    scd = dev(sc)
    for K in sorted({0, 1, 2, Nv // 3, int(np.ceil(0.3 * Nv)), Nv - 1, Nv, Nv + 9}):
        ref = oracle.topk(sc, K)
        k = min(K, Nv)
        out = torch.full((B, max(k, 1)), -1, dtype=torch.int32, device="cuda")
        qb.quota_topk_prune(scd, B, Nv, K, out)
        assert np.array_equal(host(out)[:, :k].reshape(B, k), ref), (Nv, K)
    allsame = dev(np.full((B, Nv), 0.5, np.float32))
    k = max(1, Nv // 2)
    out = torch.empty((B, k), dtype=torch.int32, device="cuda")
    qb.quota_topk_prune(allsame, B, Nv, k, out)
    assert np.array_equal(host(out), np.tile(np.arange(k, dtype=np.int32), (B, 1)))
    with pytest.raises(qb.QuotaError):
        qb.quota_topk_prune(scd, B, 8200, 3, out)
