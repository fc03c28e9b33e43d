"""GPU parity of the decode step over the pruned 4-bit KV cache (quota_attention_decode,
quota_decode_layer) against the oracle.

Teacher-forced: the oracle's attention output and SwiGLU product are injected at the tap
points, so the appended K/V codes and scales and every fp16 tensor must be BIT-EXACT.
Free-running: the attention output must be within 1e-2 relative; tensors behind a later int4
quantizer are compared statistically (one flipped code moves an input by a whole step)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl
from test_gpu_ops import _pack4, close_f16, dev, host, unpack4
from test_gpu_layer import assert_chain_report, build_layer, chain_report

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available()
    from paper_2604_17320_amd import binding
    binding.lib()
    return binding


def fill_cache(cache, c, length):
    """Loads oracle cache arrays (int8 codes [B, L, d], fp16 scales) into a KVCache4."""
    cache.k_codes[:, :length] = dev(_pack4(c["kc"]))
    cache.v_codes[:, :length] = dev(_pack4(c["vc"]))
    cache.k_scales[:, :length] = dev(c["ks"])
    cache.v_scales[:, :length] = dev(c["vs"])
    cache.desc.len = length


def random_cache(seed, B, L, H, dh):
    r = wl.rng(seed, "cache")
    k = (r.standard_normal((B * L, H * dh)) * 1.5).astype(np.float16)
    v = r.standard_normal((B * L, H * dh)).astype(np.float16)
    kc, ks, _ = oracle.kv_quant(k)
    vc, vs, _ = oracle.kv_quant(v)
    sh = lambda a: a.reshape(B, L, -1)
    return dict(kc=sh(kc), ks=sh(ks), vc=sh(vc), vs=sh(vs))


@pytest.mark.parametrize("B,L,H,dh", [(1, 1, 2, 64), (2, 37, 4, 64), (3, 300, 8, 128), (16, 366, 32, 128),
                                      (1, 2049, 2, 128)])
def test_attention_decode(qb, B, L, H, dh):
    from paper_2604_17320_amd.model import KVCache4
    c = random_cache(5, B, L, H, dh)
    q = wl.rng(6, "q").standard_normal((B, H * dh)).astype(np.float16)
    ref = oracle.decode_attention(q, c["kc"], c["ks"], c["vc"], c["vs"], H, dh)
    cache = KVCache4(B, L + 5, H, dh)
    fill_cache(cache, c, L)
    o = torch.zeros((B, H * dh), dtype=torch.float16, device="cuda")
    qb.quota_attention_decode(dev(q), cache.desc, o)
    assert close_f16(host(o), ref)


def test_attention_decode_errors(qb):
    from paper_2604_17320_amd.model import KVCache4
    cache = KVCache4(1, 8, 2, 64)
    q = torch.zeros((1, 128), dtype=torch.float16, device="cuda")
    o = torch.zeros_like(q)
    with pytest.raises(qb.QuotaError) as e:          # empty cache: nothing to attend over
        qb.quota_attention_decode(q, cache.desc, o)
    assert e.value.code == qb.ERR_INVALID_ARG
    big = KVCache4(1, 8200, 2, 64)
    big.desc.len = 8193
    with pytest.raises(qb.QuotaError) as e:
        qb.quota_attention_decode(q, big.desc, o)
    assert e.value.code == qb.ERR_SHAPE


def run_decode(qb, L, shape, x, pos, cache_arrays, inject=None):
    from paper_2604_17320_amd.model import KVCache4, make_taps
    B, d, F = x.shape[0], shape.d, shape.F
    Lc = cache_arrays["kc"].shape[1]
    cache = KVCache4(B, Lc + 4, shape.H, shape.dh)
    fill_cache(cache, cache_arrays, Lc)
    t = lambda shp: torch.zeros(shp, dtype=torch.float16, device="cuda")
    out = dict(qkv=t((B, 3 * d)), q_rot=t((B, d)), o=t((B, d)), x1=t((B, d)), gu=t((B, 2 * F)), z=t((B, F)))
    taps, keep = dict(out), []
    for name, arr in (inject or {}).items():
        keep.append(dev(arr))
        taps["inject_" + name] = keep[-1]
    x_out = t((B, d))
    ws = torch.empty(L.decode_workspace_bytes(B), dtype=torch.uint8, device="cuda")
    L.decode(dev(x), dev(pos), cache, x_out, ws, make_taps(**taps))
    res = {k: host(v) for k, v in out.items()}
    res.update(x_next=host(x_out), cache_len=cache.len,
               kc=unpack4(host(cache.k_codes)[:, Lc]), vc=unpack4(host(cache.v_codes)[:, Lc]),
               ks=host(cache.k_scales)[:, Lc], vs=host(cache.v_scales)[:, Lc],
               kc_old=unpack4(host(cache.k_codes)[:, :Lc]))
    return res


def eq16(a, b):
    return np.array_equal(np.ascontiguousarray(a).view(np.uint16), np.ascontiguousarray(b).view(np.uint16))


def check_decode(qb, shape, seed, K, steps=2):
    """Prefill (oracle) -> pruned cache -> `steps` decode steps, each checked teacher-forced and free-running."""
    W, L, cos, sin = build_layer(shape, seed, gamma_random=True)
    B, N, d = shape.B, shape.N, shape.d
    x, pos = wl.hidden_state(shape, seed), wl.positions(shape)
    pre = oracle.prefill_layer(W, x, pos, B, N, shape.vis_begin, shape.Nv, K, cos, sin, prune_mid=True)
    cache = oracle.cache_from_prefill(pre, B)
    r = wl.rng(seed, "decode-x")
    for step in range(steps):
        xn = r.standard_normal((B, d)).astype(np.float16)
        pn = np.full(B, N + step, np.int32)                   # original position id of the new token
        ref = oracle.decode_layer(W, xn, pn, cache, cos, sin)
        got = run_decode(qb, L, shape, xn, pn, cache, dict(o=ref["o"], z=ref["z"]))
        assert got["cache_len"] == cache["kc"].shape[1] + 1
        assert eq16(got["qkv"], ref["qkv"]) and eq16(got["q_rot"], ref["q"])
        assert np.array_equal(got["kc"], ref["kc"]) and np.array_equal(got["vc"], ref["vc"])
        assert eq16(got["ks"], ref["ks"]) and eq16(got["vs"], ref["vs"])
        assert np.array_equal(got["kc_old"], cache["kc"])     # earlier rows untouched
        assert eq16(got["x1"], ref["x1"]) and eq16(got["gu"], ref["gu"]) and eq16(got["x_next"], ref["x_next"])
        assert close_f16(got["o"], ref["o"])                  # the library's own attention, dumped by the same run
        free = run_decode(qb, L, shape, xn, pn, cache)
        assert close_f16(free["o"], ref["o"])
        rep = chain_report(W, free, ref)                      # int4 code flips behind the attention output
        print("decode free-running report:", rep)
        assert_chain_report(rep)
        cache = ref["cache"]


def test_decode_layer_small(qb):
    check_decode(qb, wl.CONFIGS[0], 0, 19, steps=3)


def test_decode_layer_small_batch_prefix(qb):
    base = wl.CONFIGS[0]
    shape = wl.Shape("dec_b3", d=base.d, H=base.H, F=base.F, layers=1, B=3, Nv=base.Nv, Nt=9,
                     n_outlier=base.n_outlier, vis_begin=2)
    check_decode(qb, shape, 1, 7, steps=2)


def test_decode_layer_7b_shape(qb):
    """7B-shaped layer, batch 4, cache pruned to 30 % of 576 visual tokens plus 64 text tokens."""
    base = wl.CONFIGS[1]
    shape = wl.Shape("dec_7b", d=base.d, H=base.H, F=base.F, layers=1, B=4, Nv=96, Nt=16,
                     n_outlier=base.n_outlier, vis_begin=0)
    check_decode(qb, shape, 2, 29, steps=2)


def test_decode_layer_errors(qb):
    from paper_2604_17320_amd.model import KVCache4
    shape = wl.CONFIGS[0]
    W, L, cos, sin = build_layer(shape, 1)
    x = torch.zeros((1, shape.d), dtype=torch.float16, device="cuda")
    pos = torch.zeros((1,), dtype=torch.int32, device="cuda")
    ws = torch.empty(L.decode_workspace_bytes(1), dtype=torch.uint8, device="cuda")
    full = KVCache4(1, 4, shape.H, shape.dh)
    full.desc.len = 4
    with pytest.raises(qb.QuotaError) as e:
        L.decode(x, pos, full, torch.empty_like(x), ws)
    assert e.value.code == qb.ERR_CAPACITY and full.len == 4
    wrong = KVCache4(2, 8, shape.H, shape.dh)
    with pytest.raises(qb.QuotaError) as e:
        L.decode(x, pos, wrong, torch.empty_like(x), ws)
    assert e.value.code == qb.ERR_SHAPE
