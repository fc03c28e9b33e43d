"""GPU parity with grouped-query attention (fewer K/V heads than query heads, as in the paper's
second model family): the attention entry points on their own, then a whole layer (prefill,
teacher-forced bit-exact, the narrower 4-bit cache) and decode steps over that cache."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl
from test_gpu_ops import _act, _pack4, close_f16, dev, host, unpack4
from test_gpu_layer import assert_chain_report, chain_report
from test_gpu_decode import eq16, fill_cache

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available()
    from paper_2604_17320_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("B,N,H,Hkv,dh,vb,Nv", [(2, 150, 6, 2, 64, 3, 100), (1, 300, 8, 2, 128, 0, 260),
                                                 (1, 70, 4, 1, 128, 0, 50)])
def test_attention_prefill_gqa(qb, B, N, H, Hkv, dh, vb, Nv):
    q = _act(B * N, H * dh, 91, 1.0)
    _, _, khat = oracle.kv_quant(_act(B * N, Hkv * dh, 92, 1.0))
    _, _, vhat = oracle.kv_quant(_act(B * N, Hkv * dh, 93, 1.0))
    o_ref, ci_ref, cv_ref = oracle.attention(q, khat, vhat, B, N, H, dh, vb, Nv, Hkv=Hkv)
    o = torch.empty((B * N, H * dh), dtype=torch.float16, device="cuda")
    ci, cv = (torch.zeros((B, Nv), dtype=torch.float32, device="cuda") for _ in range(2))
    ws = torch.empty(qb.quota_attention_workspace_bytes(B, N, H, dh), dtype=torch.uint8, device="cuda")
    qb.quota_attention_prefill_gqa(dev(q), dev(khat), dev(vhat), B, N, H, Hkv, dh, vb, Nv, o, ci, cv, ws)
    assert close_f16(host(o), o_ref)
    assert np.allclose(host(ci), ci_ref, rtol=2e-5, atol=1e-7) and np.allclose(host(cv), cv_ref, rtol=2e-5, atol=1e-7)


def test_attention_decode_gqa(qb):
    from paper_2604_17320_amd.model import KVCache4
    B, L, Hq, Hkv, dh = 3, 210, 8, 2, 128
    r = wl.rng(94, "gqa-dec")
    kc, ks, _ = oracle.kv_quant((r.standard_normal((B * L, Hkv * dh)) * 1.5).astype(np.float16))
    vc, vs, _ = oracle.kv_quant(r.standard_normal((B * L, Hkv * dh)).astype(np.float16))
    sh = lambda a: a.reshape(B, L, -1)
    c = dict(kc=sh(kc), ks=sh(ks), vc=sh(vc), vs=sh(vs))
    q = r.standard_normal((B, Hq * dh)).astype(np.float16)
    ref = oracle.decode_attention(q, c["kc"], c["ks"], c["vc"], c["vs"], Hq, dh, Hkv)
    cache = KVCache4(B, L + 2, Hkv, dh)
    fill_cache(cache, c, L)
    o = torch.zeros((B, Hq * dh), dtype=torch.float16, device="cuda")
    qb.quota_attention_decode_gqa(dev(q), Hq, cache.desc, o)
    assert close_f16(host(o), ref)
    with pytest.raises(qb.QuotaError) as e:
        qb.quota_attention_decode_gqa(dev(q), 7, cache.desc, o)       # 7 query heads over 2 K/V heads
    assert e.value.code == qb.ERR_SHAPE


@pytest.mark.parametrize("B,L,Hq,Hkv,dh", [
    (2, 700, 28, 4, 128),      # 7 query heads per K/V head: the last workgroup of a head serves one query head
    (3, 513, 6, 3, 64),        # head_dim 64, one row past a 512-row tile, a grid that is no multiple of 8
    (1, 512, 4, 1, 128),       # exactly one tile, one K/V head
    (5, 1100, 10, 5, 128),     # three tiles of the running softmax
])
def test_attention_decode_gqa_shapes(qb, B, L, Hq, Hkv, dh):
    """Grouped heads through the decode attention's workgroup layout: one workgroup per (sequence,
    K/V head, pair of query heads), dealt to the XCDs in contiguous ranges."""
    from paper_2604_17320_amd.model import KVCache4
    r = wl.rng(95, "gqa-dec", B, L, Hq)
    kc, ks, _ = oracle.kv_quant((r.standard_normal((B * L, Hkv * dh)) * 1.5).astype(np.float16))
    vc, vs, _ = oracle.kv_quant(r.standard_normal((B * L, Hkv * dh)).astype(np.float16))
    sh = lambda a: a.reshape(B, L, -1)
    c = dict(kc=sh(kc), ks=sh(ks), vc=sh(vc), vs=sh(vs))
    q = r.standard_normal((B, Hq * dh)).astype(np.float16)
    ref = oracle.decode_attention(q, c["kc"], c["ks"], c["vc"], c["vs"], Hq, dh, Hkv)
    cache = KVCache4(B, L + 3, Hkv, dh)
    fill_cache(cache, c, L)
    o = torch.full((B, Hq * dh), float("nan"), dtype=torch.float16, device="cuda")     # every output must be written
    qb.quota_attention_decode_gqa(dev(q), Hq, cache.desc, o)
    assert close_f16(host(o), ref)


def build_gqa_layer(d, H, Hkv, dh, F, seed, n_pos):
    from paper_2604_17320_amd.model import PackedLinear, PrefillLayer
    r = wl.rng(seed, "gqa-layer")
    mk = lambda n, k: oracle.quantize_weights((r.standard_normal((n, k)) * 0.02).astype(np.float32))
    q = dict(qkv=mk(d + 2 * Hkv * dh, d), o=mk(d, d), gu=mk(2 * F, d), down=mk(d, F))
    g1 = r.uniform(0.7, 1.3, d).astype(np.float32)
    g2 = r.uniform(0.7, 1.3, d).astype(np.float32)
    W = oracle.LayerWeights(qkv=q["qkv"], o=q["o"], gu=q["gu"], down=q["down"], gamma1=g1, gamma2=g2, eps=1e-5,
                            H=H, dh=dh, F=F, Hkv=Hkv)
    cos, sin = wl.rope_tables(dh, n_pos)
    lin = {k: PackedLinear.from_codes(dev(c), dev(s)) for k, (c, s) in q.items()}
    L = PrefillLayer(H, dh, F, lin["qkv"], lin["o"], lin["gu"], lin["down"], dev(g1), dev(g2), 1e-5, dev(cos),
                     dev(sin), Hkv=Hkv)
    return W, L, cos, sin


@pytest.mark.parametrize("d,H,Hkv,dh,F,B,Nv,Nt,K", [(512, 8, 2, 64, 1376, 2, 64, 16, 19),
                                                    (1024, 8, 2, 128, 2048, 1, 200, 24, 60),
                                                    (256, 4, 1, 64, 160, 2, 40, 8, 11)])   # K/V width 64: unfused path
def test_layer_gqa_prefill_then_decode(qb, d, H, Hkv, dh, F, B, Nv, Nt, K):
    from paper_2604_17320_amd.model import KVCache4, make_taps
    N, dkv = Nv + Nt, Hkv * dh
    shape = wl.Shape("gqa", d=d, H=H, F=F, layers=1, B=B, Nv=Nv, Nt=Nt, n_outlier=4, vis_begin=0)
    W, L, cos, sin = build_gqa_layer(d, H, Hkv, dh, F, 7, N + 8)
    x, pos = wl.hidden_state(shape, 7), wl.positions(shape)
    ref = oracle.prefill_layer(W, x, pos, B, N, 0, Nv, K, cos, sin, prune_mid=True)
    n_keep = N - Nv + K
    t16 = lambda *shp: torch.zeros(shp, dtype=torch.float16, device="cuda")
    out = dict(qkv=t16(B * N, d + 2 * dkv), q_rot=t16(B * N, d), o=t16(B * N, d), x1=t16(B * n_keep, d),
               gu=t16(B * n_keep, 2 * F), score=torch.zeros((B, Nv), dtype=torch.float32, device="cuda"),
               keep_idx=torch.zeros((B, K), dtype=torch.int32, device="cuda"))
    inj = {k: dev(ref[k]) for k in ("o", "z", "cm_inter", "cm_intra")}
    taps = make_taps(**out, inject_o=inj["o"], inject_z=inj["z"], inject_cm_inter=inj["cm_inter"],
                     inject_cm_intra=inj["cm_intra"])
    cache = KVCache4(B, n_keep + 4, Hkv, dh)
    x_out, pos_out = t16(B * n_keep, d), torch.zeros((B * n_keep,), dtype=torch.int32, device="cuda")
    ws = torch.empty(L.workspace_bytes(B, N), dtype=torch.uint8, device="cuda")
    xd, pd = dev(x), dev(pos)
    st = qb.State(B, N, 0, Nv, xd.data_ptr(), pd.data_ptr(), x_out.data_ptr(), pos_out.data_ptr())
    qb.quota_prefill_layer(L.desc, st, K, qb.quota_score_params_default(), cache.desc, taps, ws)
    assert eq16(host(out["qkv"]), ref["qkv"]) and eq16(host(out["q_rot"]), ref["q"])
    assert np.array_equal(host(out["score"]), ref["score"]) and np.array_equal(host(out["keep_idx"]), ref["keep_idx"])
    assert cache.len == n_keep and cache.k_codes.shape[-1] == dkv // 2
    assert np.array_equal(unpack4(host(cache.k_codes)[:, :n_keep]).reshape(B * n_keep, dkv), ref["cache_kc"])
    assert np.array_equal(unpack4(host(cache.v_codes)[:, :n_keep]).reshape(B * n_keep, dkv), ref["cache_vc"])
    assert eq16(host(cache.k_scales)[:, :n_keep].reshape(B * n_keep, -1), ref["cache_ks"])
    assert eq16(host(out["x1"]), ref["x1"]) and eq16(host(out["gu"]), ref["gu"]) and eq16(host(x_out), ref["x_next"])
    assert close_f16(host(out["o"]), ref["o"])              # the library's own attention, dumped by the same run

    # decode over the pruned, narrower cache
    ocache = oracle.cache_from_prefill(ref, B)
    r = wl.rng(8, "gqa-dec-x")
    dws = torch.empty(L.decode_workspace_bytes(B), dtype=torch.uint8, device="cuda")
    for step in range(2):
        xn = r.standard_normal((B, d)).astype(np.float16)
        pn = np.full(B, N + step, np.int32)
        dref = oracle.decode_layer(W, xn, pn, ocache, cos, sin)
        dout = dict(q_rot=t16(B, d), o=t16(B, d), x1=t16(B, d))
        di = {k: dev(dref[k]) for k in ("o", "z")}
        y = t16(B, d)
        Lc = cache.len
        L.decode(dev(xn), dev(pn), cache, y, dws, make_taps(**dout, inject_o=di["o"], inject_z=di["z"]))
        assert cache.len == Lc + 1
        assert eq16(host(dout["q_rot"]), dref["q"]) and eq16(host(dout["x1"]), dref["x1"]) and eq16(host(y), dref["x_next"])
        assert np.array_equal(unpack4(host(cache.k_codes)[:, Lc]), dref["kc"])
        assert eq16(host(cache.v_scales)[:, Lc], dref["vs"])
        assert close_f16(host(dout["o"]), dref["o"])
        free = t16(B, d)
        fo = dict(o=t16(B, d), x1=t16(B, d), gu=t16(B, 2 * F), z=t16(B, F))
        cache.desc.len = Lc                                  # same step again, free-running
        L.decode(dev(xn), dev(pn), cache, free, dws, make_taps(**fo))
        rep = chain_report(W, dict({k_: host(v_) for k_, v_ in fo.items()}, x_next=host(free)), dref)
        print("gqa decode free-running report:", rep)
        assert_chain_report(rep)
        ocache = dref["cache"]


def test_layer_qwen25_vl_7b_shape(qb):
    """One layer at the shape of the paper's second model family (Qwen2.5-VL-7B language model:
    d = 3584, 28 query heads over 4 K/V heads of 128, SwiGLU FFN 18944 -- wider than the 16384 columns
    one workgroup row used to hold), 300 visual + 20 text tokens, budget 90 (30 %): prefill
    teacher-forced bit-exact incl. the narrow 4-bit cache; then the same layer as a layer outside the
    candidate set (supplementary: pruning at layers 8-12 only), which must keep every token."""
    from paper_2604_17320_amd.model import KVCache4, make_taps
    d, H, Hkv, dh, F, B, Nv, Nt, K = 3584, 28, 4, 128, 18944, 1, 300, 20, 90
    N, dkv = Nv + Nt, Hkv * dh
    W, L, cos, sin = build_gqa_layer(d, H, Hkv, dh, F, 21, N + 8)
    shape = wl.Shape("qwen", d=d, H=H, F=F, layers=1, B=B, Nv=Nv, Nt=Nt, n_outlier=36, vis_begin=0)
    x, pos = wl.hidden_state(shape, 21), wl.positions(shape)
    t16 = lambda *shp: torch.zeros(shp, dtype=torch.float16, device="cuda")
    for K_l, K_or in ((K, K), (qb.KEEP_ALL, Nv)):
        print("qwen-shaped layer, K_l =", K_l, flush=True)
        ref = oracle.prefill_layer(W, x, pos, B, N, 0, Nv, K_or, cos, sin, prune_mid=True)
        n_keep = N - Nv + K_or
        out = dict(qkv=t16(B * N, d + 2 * dkv), q_rot=t16(B * N, d), o=t16(B * N, d), x1=t16(B * n_keep, d),
                   gu=t16(B * n_keep, 2 * F), keep_idx=torch.full((B, K_or), -1, dtype=torch.int32, device="cuda"))
        inj = {k: dev(ref[k]) for k in ("o", "z", "cm_inter", "cm_intra")}
        taps = make_taps(**out, inject_o=inj["o"], inject_z=inj["z"], inject_cm_inter=inj["cm_inter"],
                         inject_cm_intra=inj["cm_intra"])
        cache = KVCache4(B, n_keep + 2, Hkv, dh)
        x_out, pos_out = t16(B * n_keep, d), torch.zeros((B * n_keep,), dtype=torch.int32, device="cuda")
        ws = torch.empty(L.workspace_bytes(B, N), dtype=torch.uint8, device="cuda")
        xd, pd = dev(x), dev(pos)
        st = qb.State(B, N, 0, Nv, xd.data_ptr(), pd.data_ptr(), x_out.data_ptr(), pos_out.data_ptr())
        qb.quota_prefill_layer(L.desc, st, K_l, qb.quota_score_params_default(), cache.desc, taps, ws)
        assert (st.N, st.Nv, cache.len) == (n_keep, K_or, n_keep)
        assert eq16(host(out["qkv"]), ref["qkv"]) and eq16(host(out["q_rot"]), ref["q"])
        if K_l == qb.KEEP_ALL:
            assert np.all(host(out["keep_idx"]) == -1)                     # no selection ran
        else:
            assert np.array_equal(host(out["keep_idx"]), ref["keep_idx"])
        assert np.array_equal(host(pos_out), ref["pos_next"])
        assert np.array_equal(unpack4(host(cache.k_codes)[:, :n_keep]).reshape(B * n_keep, dkv), ref["cache_kc"])
        assert np.array_equal(unpack4(host(cache.v_codes)[:, :n_keep]).reshape(B * n_keep, dkv), ref["cache_vc"])
        assert eq16(host(cache.v_scales)[:, :n_keep].reshape(B * n_keep, -1), ref["cache_vs"])
        assert eq16(host(out["x1"]), ref["x1"]) and eq16(host(out["gu"]), ref["gu"]) and eq16(host(x_out), ref["x_next"])
        assert close_f16(host(out["o"]), ref["o"])
