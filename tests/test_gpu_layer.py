"""GPU parity of quota_prefill_layer against the oracle's layer composite.

Two modes.  Teacher-forced: the oracle's attention output, column masses and
SwiGLU product are injected at the library's tap points, so every integer
output and every fp16 tensor downstream must then be BIT-EXACT.  Free-running:
the GPU consumes its own floats; fp16 tensors must be within 1e-2 relative,
scores within 1e-5 relative (after the column masses' own tolerance), and the
kept index set must equal the oracle's except where the oracle's score gap
across the cut is below that tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl
from test_gpu_ops import close_f16, dev, host, unpack4

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available()
    from paper_2604_17320_amd import binding
    binding.lib()
    return binding


def build_layer(shape, seed, gamma_random=False):
    from paper_2604_17320_amd.model import PackedLinear, PrefillLayer
    fw = wl.fp_weights(shape, seed)
    q = {k: oracle.quantize_weights(v) for k, v in fw.items()}
    d = shape.d
    if gamma_random:
        g1 = wl.rng(seed, "g1").uniform(0.7, 1.3, d).astype(np.float32)
        g2 = wl.rng(seed, "g2").uniform(0.7, 1.3, d).astype(np.float32)
    else:
        g1 = np.ones(d, np.float32)
        g2 = np.ones(d, np.float32)
    W = oracle.LayerWeights(qkv=q["qkv"], o=q["o"], gu=q["gu"], down=q["down"], gamma1=g1, gamma2=g2,
                            eps=1e-5, H=shape.H, dh=shape.dh, F=shape.F)
    cos, sin = wl.rope_tables(shape.dh, shape.N + 8)
    lin = {k: PackedLinear.from_codes(dev(c), dev(s)) for k, (c, s) in q.items()}
    L = PrefillLayer(shape.H, shape.dh, shape.F, lin["qkv"], lin["o"], lin["gu"], lin["down"], dev(g1),
                     dev(g2), 1e-5, dev(cos), dev(sin))
    return W, L, cos, sin


def run_gpu(qb, L, shape, x, pos, K, inject=None):
    from paper_2604_17320_amd.model import KVCache4, make_taps
    B, N, Nv, vb, d, F = shape.B, shape.N, shape.Nv, shape.vis_begin, shape.d, shape.F
    k = min(K, Nv)
    n_keep = N - Nv + k
    t = lambda shp, dt: torch.zeros(shp, dtype=dt, device="cuda")
    out = dict(qkv=t((B * N, 3 * d), torch.float16), q_rot=t((B * N, d), torch.float16),
               o=t((B * N, d), torch.float16), sumsq=t((B, max(Nv, 1)), torch.float32),
               ressq=t((B, max(Nv, 1)), torch.float32), cm_inter=t((B, max(Nv, 1)), torch.float32),
               cm_intra=t((B, max(Nv, 1)), torch.float32), score=t((B, max(Nv, 1)), torch.float32),
               keep_idx=t((B, max(k, 1)), torch.int32), rows=t((B, max(n_keep, 1)), torch.int32),
               x1=t((max(B * n_keep, 1), d), torch.float16), gu=t((max(B * n_keep, 1), 2 * F), torch.float16),
               z=t((max(B * n_keep, 1), F), torch.float16))
    keep_alive = []
    taps = dict(out)
    if inject:
        for name, arr in inject.items():
            tens = dev(arr)
            keep_alive.append(tens)
            taps["inject_" + name] = tens
    cache = KVCache4(B, n_keep + 3, shape.H, shape.dh)
    x_out = t((max(B * n_keep, 1), d), torch.float16)
    pos_out = t((max(B * n_keep, 1),), torch.int32)
    ws = torch.empty(L.workspace_bytes(B, N), dtype=torch.uint8, device="cuda")
    xd, pd = dev(x), dev(pos)
    st = qb.State(B, N, vb, Nv, xd.data_ptr(), pd.data_ptr(), x_out.data_ptr(), pos_out.data_ptr())
    qb.quota_prefill_layer(L.desc, st, K, qb.quota_score_params_default(), cache.desc, make_taps(**taps), ws)
    res = {k_: host(v) for k_, v in out.items()}
    res.update(x_next=host(x_out), pos_next=host(pos_out), N=st.N, Nv=st.Nv, cache_len=cache.len,
               cache_kc=unpack4(host(cache.k_codes)[:, :n_keep]).reshape(B * n_keep, d),
               cache_vc=unpack4(host(cache.v_codes)[:, :n_keep]).reshape(B * n_keep, d),
               cache_ks=host(cache.k_scales)[:, :n_keep].reshape(B * n_keep, -1),
               cache_vs=host(cache.v_scales)[:, :n_keep].reshape(B * n_keep, -1))
    return res


def assert_teacher_forced_exact(ref, got, shape, K):
    B, Nv = shape.B, shape.Nv
    k = min(K, Nv)
    n_keep = shape.N - Nv + k
    eq16 = lambda a, b: np.array_equal(np.ascontiguousarray(a).view(np.uint16), np.ascontiguousarray(b).view(np.uint16))
    assert eq16(got["qkv"], ref["qkv"]) and eq16(got["q_rot"], ref["q"])
    if Nv:
        assert np.array_equal(got["sumsq"], ref["sumsq"]) and np.array_equal(got["ressq"], ref["ressq"])
        assert np.array_equal(got["score"], ref["score"])
    assert got["N"] == n_keep and got["Nv"] == k and got["cache_len"] == n_keep
    if k:
        assert np.array_equal(got["keep_idx"][:, :k], ref["keep_idx"])
    if n_keep:
        assert np.array_equal(got["rows"], ref["rows"])
        assert np.array_equal(got["pos_next"][: B * n_keep], ref["pos_next"])
        assert np.array_equal(got["cache_kc"], ref["cache_kc"]) and np.array_equal(got["cache_vc"], ref["cache_vc"])
        assert eq16(got["cache_ks"], ref["cache_ks"]) and eq16(got["cache_vs"], ref["cache_vs"])
        assert eq16(got["x1"], ref["x1"]) and eq16(got["gu"], ref["gu"])
        assert eq16(got["x_next"][: B * n_keep], ref["x_next"])


CASES = [
    # name, shape overrides, K
    ("c1", dict(), 19),
    ("many_rows", dict(B=8, Nv=384, Nt=16), 100),      # 3200 rows: the tile choices of mid-sized launches
    ("c1_k20", dict(), 20),
    ("keep_all", dict(), 999),
    ("keep_none", dict(), 0),
    ("batch2_prefix", dict(B=2, vis_begin=3, Nt=9), 19),
    ("no_visual", dict(Nv=0, Nt=40), 5),
    ("long_visual_prefix", dict(Nv=4100, Nt=28), 1000),   # more scored tokens than fit the default LDS limit of a launch
]


@pytest.mark.parametrize("name,over,K", CASES, ids=[c[0] for c in CASES])
def test_layer_small_teacher_forced(qb, name, over, K):
    base = wl.CONFIGS[0]
    kw = dict(name=name, d=base.d, H=base.H, F=base.F, layers=1, B=base.B, Nv=base.Nv, Nt=base.Nt,
              n_outlier=base.n_outlier, vis_begin=0)
    kw.update(over)
    shape = wl.Shape(**kw)
    W, L, cos, sin = build_layer(shape, 0, gamma_random=True)
    x, pos = wl.hidden_state(shape, 0), wl.positions(shape)
    ref = oracle.prefill_layer(W, x, pos, shape.B, shape.N, shape.vis_begin, shape.Nv, K, cos, sin,
                               prune_mid=True)
    inject = dict(o=ref["o"], z=ref["z"])
    if shape.Nv:
        inject.update(cm_inter=ref["cm_inter"], cm_intra=ref["cm_intra"])
    got = run_gpu(qb, L, shape, x, pos, K, inject)
    assert_teacher_forced_exact(ref, got, shape, K)
    # the GPU's own attention / cue / SwiGLU outputs, dumped by the same run, within tolerance
    assert close_f16(got["o"], ref["o"])
    if shape.Nv:
        assert np.allclose(got["cm_inter"], ref["cm_inter"], rtol=2e-5, atol=1e-7)
        assert np.allclose(got["cm_intra"], ref["cm_intra"], rtol=2e-5, atol=1e-7)


def close_f32(a, b, rtol=1e-5):
    """fp32 contract: |a - b| <= rtol * max(|b|, rms(b)), element by element."""
    a, b = a.astype(np.float64), b.astype(np.float64)
    rms = np.sqrt((b ** 2).mean()) if b.size else 0.0
    return bool(np.all(np.abs(a - b) <= rtol * np.maximum(np.abs(b), rms)))


# Share of int4 codes that may differ at a quantizer of a free-running chain.  A code flips when the
# two sides' inputs fall on different sides of a rounding boundary: inputs that differ by one fp16
# ulp (2^-11 relative) do so with probability ~ |x| / step * 2^-11 per element (a few 1e-3 at most);
# a row whose absmax element moved re-scales the whole row, which moves more codes of that row.
# Flips then feed the next quantizer through an exact GEMM and a row normalisation or a product.
FLIP_BOUND = dict(qa2=2e-3, qa3=2e-3, qa4=5e-3)      # measured: up to 3.3e-4, 1e-5, 8.5e-4


def free_running_report(ref, got, shape, K, W):
    """Where a free-running GPU chain and the oracle part ways, quantizer by quantizer: the int4
    codes each quantizer WOULD emit for the GPU's tensor (oracle quantizer applied to it -- the GPU
    quantizers equal it bit for bit on equal inputs) against the oracle's own codes.  Rows are the
    kept rows common to both sides."""
    B, N, Nv = shape.B, shape.N, shape.Nv
    k = min(K, Nv)
    n_keep = N - Nv + k
    g_rows, r_rows = got["rows"].reshape(B, n_keep), ref["rows"].reshape(B, n_keep)
    gi, ri = [], []                                    # positions (in the compacted tensors) of the common rows
    for b in range(B):
        common = np.intersect1d(g_rows[b], r_rows[b])
        gi.append(b * n_keep + np.searchsorted(g_rows[b], common))
        ri.append(b * n_keep + np.searchsorted(r_rows[b], common))
    gi, ri = np.concatenate(gi), np.concatenate(ri)
    flat_g = (np.arange(B)[:, None] * N + g_rows).reshape(-1)[gi]
    flat_r = (np.arange(B)[:, None] * N + r_rows).reshape(-1)[ri]
    rep = chain_report(W, dict(o=got["o"][flat_g], x1=got["x1"][gi], gu=got["gu"][gi], z=got["z"][gi], x_next=got["x_next"][gi]),
                       dict(o=ref["o"][flat_r], x1=ref["x1"][ri], gu=ref["gu"][ri], z=ref["z"][ri], x_next=ref["x_next"][ri]))
    rep["rows"] = len(gi)
    return rep, gi, ri


def chain_report(W, g, r):
    """Token-wise rest of the block, GPU tensors `g` against oracle tensors `r` (same rows): share of
    int4 codes that differ at the three quantizers (in front of O, gate/up, down), and whether every
    row whose quantized input (codes and scale) agrees is bit-exact behind the GEMM that follows."""
    rep = {}

    def codes(t):
        q, s_, _, _ = oracle.quantize_act(t)
        return q, s_

    def cmp(name, tg, tr):
        (qg, sg), (qr, sr) = codes(tg), codes(tr)
        rep[name] = float((qg != qr).mean())
        return np.all(qg == qr, axis=1) & (sg == sr)

    same2 = cmp("qa2", g["o"], r["o"])
    same3 = cmp("qa3", oracle.rmsnorm(g["x1"], W.gamma2, W.eps), oracle.rmsnorm(r["x1"], W.gamma2, W.eps))
    same4 = cmp("qa4", g["z"], r["z"])
    eq_rows = lambda a, b_: np.all(np.ascontiguousarray(a).view(np.uint16) == np.ascontiguousarray(b_).view(np.uint16), axis=1)
    x1_eq, gu_eq, xn_eq = eq_rows(g["x1"], r["x1"]), eq_rows(g["gu"], r["gu"]), eq_rows(g["x_next"], r["x_next"])
    # a GEMM is exact, so a row whose quantized input (codes and scale) and residual agree must agree bit for bit
    rep["x1_rows_checked"], rep["x1_ok"] = int(same2.sum()), bool(np.all(x1_eq[same2]))
    rep["gu_rows_checked"], rep["gu_ok"] = int(same3.sum()), bool(np.all(gu_eq[same3]))
    ok4 = same4 & x1_eq
    rep["xn_rows_checked"], rep["xn_ok"] = int(ok4.sum()), bool(np.all(xn_eq[ok4]))
    rep["rel_rms"] = dict(x1=rel_rms(g["x1"], r["x1"]), gu=rel_rms(g["gu"], r["gu"]), x_next=rel_rms(g["x_next"], r["x_next"]))
    return rep


def assert_chain_report(rep):
    for q in ("qa2", "qa3", "qa4"):
        assert rep[q] <= FLIP_BOUND[q], (q, rep[q])
    assert rep["x1_ok"] and rep["gu_ok"] and rep["xn_ok"], rep
    assert rep["rel_rms"]["x1"] < 1e-2 and rep["rel_rms"]["gu"] < 5e-2 and rep["rel_rms"]["x_next"] < 5e-2


def check_free_running(ref, got, shape, K, W):
    """Free-running chain (the GPU consumes its own floats) against the oracle.  fp16 tensors in front
    of the first re-quantization within 1e-2, scores within 1e-5 relative; kept sets equal except
    for tokens whose oracle score lies within that score tolerance of the cut (each printed); K/V
    codes of the common rows bit-exact.  Behind the attention output every tensor sits behind an
    int4 quantizer, where a one-ulp input difference can move a value by a whole quantization step:
    an element-wise fp16 bound cannot hold there (an earlier version of this test asserted it at the
    7B shape and failed on x1 and gu), so what is asserted instead is (a) the share of flipped int4
    codes at each quantizer stays under a stated bound and (b) every row whose quantized input did
    not flip is bit-exact behind the following GEMM.  The relative rms is reported as a secondary
    figure."""
    B, Nv = shape.B, shape.Nv
    k = min(K, Nv)
    n_keep = shape.N - Nv + k
    assert np.array_equal(np.ascontiguousarray(got["qkv"]).view(np.uint16), ref["qkv"].view(np.uint16))
    assert close_f16(got["o"], ref["o"])
    if Nv:
        assert close_f32(got["score"], ref["score"]), np.abs(got["score"] - ref["score"]).max()
    # index sets: equal, except swaps among tokens whose oracle scores are within the score tolerance of the cut
    for b in range(B):
        a, r = set(got["keep_idx"][b, :k].tolist()), set(ref["keep_idx"][b].tolist())
        if a != r:
            sc = ref["score"][b].astype(np.float64)
            cut = np.sort(sc)[::-1][k - 1]
            tol = 2e-5 * max(abs(cut), float(np.sqrt((sc ** 2).mean())))      # 1e-5 relative on either side
            for i in sorted(a ^ r):
                print(f"kept-set exception: sequence {b} token {i} score {sc[i]:.9g} cut {cut:.9g} gap {abs(sc[i] - cut):.3g}")
                assert abs(sc[i] - cut) <= tol, (b, i, sc[i], cut)
    if n_keep == 0:
        return None
    rep, gi, ri = free_running_report(ref, got, shape, K, W)
    print("free-running report:", rep)
    assert rep["rows"] >= B * (n_keep - 2 * 4)           # at most a few tokens swapped at the cut
    # K/V codes come from the bit-exact qkv: no float chain before them
    assert np.array_equal(got["cache_kc"][gi], ref["cache_kc"][ri]) and np.array_equal(got["cache_vc"][gi], ref["cache_vc"][ri])
    assert np.array_equal(got["pos_next"][gi], ref["pos_next"][ri])
    assert_chain_report(rep)
    assert rep["x1_rows_checked"] > 0
    return rep


def rel_rms(a, b):
    a = a.astype(np.float64)
    b = b.astype(np.float64)
    return float(np.sqrt(((a - b) ** 2).mean()) / max(np.sqrt((b ** 2).mean()), 1e-30))


def test_layer_small_free_running(qb):
    shape = wl.CONFIGS[0]
    W, L, cos, sin = build_layer(shape, 0)
    x, pos = wl.hidden_state(shape, 0), wl.positions(shape)
    for K in (19, 20):
        ref = oracle.prefill_layer(W, x, pos, 1, shape.N, 0, shape.Nv, K, cos, sin)
        got = run_gpu(qb, L, shape, x, pos, K)
        check_free_running(ref, got, shape, K, W)


def test_layer_7b_shape_full_size(qb):
    """The single 7B-shaped layer at its full size (640 tokens, keep 173), teacher-forced bit-exact and
    free-running within tolerance; the oracle needs a few tens of seconds on 8+ cores."""
    shape = wl.CONFIGS[1]
    W, L, cos, sin = build_layer(shape, 0)
    x, pos = wl.hidden_state(shape, 0), wl.positions(shape)
    K = wl.schedule_for(shape)[0]
    assert K == 173
    ref = oracle.prefill_layer(W, x, pos, 1, shape.N, 0, shape.Nv, K, cos, sin, prune_mid=True)
    got = run_gpu(qb, L, shape, x, pos, K, dict(o=ref["o"], z=ref["z"], cm_inter=ref["cm_inter"],
                                                cm_intra=ref["cm_intra"]))
    assert_teacher_forced_exact(ref, got, shape, K)
    free = run_gpu(qb, L, shape, x, pos, K)
    check_free_running(ref, free, shape, K, W)


def test_layer_errors(qb):
    from paper_2604_17320_amd.model import KVCache4
    shape = wl.CONFIGS[0]
    W, L, cos, sin = build_layer(shape, 1)
    x, pos = dev(wl.hidden_state(shape, 0)), dev(wl.positions(shape))
    x_out = torch.empty_like(x)
    pos_out = torch.empty_like(pos)
    ws = torch.empty(L.workspace_bytes(1, shape.N), dtype=torch.uint8, device="cuda")
    p = qb.quota_score_params_default()
    small = KVCache4(1, 10, shape.H, shape.dh)
    st = qb.State(1, shape.N, 0, shape.Nv, x.data_ptr(), pos.data_ptr(), x_out.data_ptr(), pos_out.data_ptr())
    with pytest.raises(qb.QuotaError) as e:
        qb.quota_prefill_layer(L.desc, st, 19, p, small.desc, None, ws)
    assert e.value.code == qb.ERR_CAPACITY and small.len == 0 and st.N == shape.N
    st_bad = qb.State(1, shape.N, 70, shape.Nv, x.data_ptr(), pos.data_ptr(), x_out.data_ptr(), pos_out.data_ptr())
    ok = KVCache4(1, 80, shape.H, shape.dh)
    with pytest.raises(qb.QuotaError) as e:
        qb.quota_prefill_layer(L.desc, st_bad, 19, p, ok.desc, None, ws)
    assert e.value.code == qb.ERR_INVALID_ARG


def test_layer_without_taps_equals_layer_with_taps(qb):
    """The benchmark runs the layer with no dump taps (the QKV projection then keeps no plain copy of
    its output); the result must be the same bits as the tapped run the parity tests check."""
    from paper_2604_17320_amd.model import KVCache4
    shape = wl.CONFIGS[0]
    W, L, cos, sin = build_layer(shape, 2)
    x, pos = wl.hidden_state(shape, 2), wl.positions(shape)
    K = 19
    tapped = run_gpu(qb, L, shape, x, pos, K)
    n_keep = shape.N - shape.Nv + K
    cache = KVCache4(1, n_keep, shape.H, shape.dh)
    x_out = torch.zeros((n_keep, shape.d), dtype=torch.float16, device="cuda")
    pos_out = torch.zeros((n_keep,), dtype=torch.int32, device="cuda")
    ws = torch.empty(L.workspace_bytes(1, shape.N), dtype=torch.uint8, device="cuda")
    xd, pd = dev(x), dev(pos)
    st = qb.State(1, shape.N, 0, shape.Nv, xd.data_ptr(), pd.data_ptr(), x_out.data_ptr(), pos_out.data_ptr())
    qb.quota_prefill_layer(L.desc, st, K, qb.quota_score_params_default(), cache.desc, None, ws)
    assert np.array_equal(host(x_out).view(np.uint16), tapped["x_next"][:n_keep].view(np.uint16))
    assert np.array_equal(host(pos_out), tapped["pos_next"][:n_keep])
    assert np.array_equal(unpack4(host(cache.k_codes)[0, :n_keep]), tapped["cache_kc"])
    assert np.array_equal(host(cache.v_scales)[0, :n_keep].view(np.uint16), tapped["cache_vs"].view(np.uint16))


@pytest.mark.parametrize("tile", [1, 2, 3, 4])
def test_layer_every_tile_with_fused_qkv_epilogue(qb, tile, pinned_gemm):
    """The QKV projection with its fused RoPE / KV-quantizer epilogue on each tile that carries it
    (and every other GEMM of the layer on the same tile), teacher-forced bit-exact."""
    pinned_gemm(tile)
    base = wl.CONFIGS[0]
    shape = wl.Shape("tile", d=base.d, H=base.H, F=base.F, layers=1, B=2, Nv=base.Nv, Nt=21,
                     n_outlier=base.n_outlier, vis_begin=0)
    W, L, cos, sin = build_layer(shape, 3, gamma_random=True)
    x, pos = wl.hidden_state(shape, 3), wl.positions(shape)
    K = 19
    ref = oracle.prefill_layer(W, x, pos, shape.B, shape.N, 0, shape.Nv, K, cos, sin, prune_mid=True)
    got = run_gpu(qb, L, shape, x, pos, K, dict(o=ref["o"], z=ref["z"], cm_inter=ref["cm_inter"],
                                                cm_intra=ref["cm_intra"]))
    assert_teacher_forced_exact(ref, got, shape, K)
