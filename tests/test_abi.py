"""CPU-side checks of the C ABI: the shared library loads, exports every function the
header declares, and its host-only logic (names, sizes, argument checks that come before
any device work) behaves as the header says.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "quota.h")
LIB = os.path.join(ROOT, "paper_2604_17320_amd", "libquota.so")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)          # comments out
    src = re.sub(r"typedef\s+struct\s+\w*\s*\{.*?\}\s*\w+\s*;", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(quota_[a-z0-9_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libquota.so is not built: run __graft_entry__.build() first")
    return C.CDLL(LIB)


def test_header_declares_the_boundary_calls():
    names = declared_functions()
    for must in ("quota_quantize_act", "quota_w4a4_gemm", "quota_score_tokens", "quota_topk_prune",
                 "quota_kv_quant_append", "quota_prefill_layer"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, f"declared in quota.h but not exported: {missing}"


def test_binding_mirrors_the_header():
    from paper_2604_17320_amd import binding
    missing = [n for n in declared_functions() if not hasattr(binding, n)]
    assert not missing, f"declared in quota.h but absent from the Python binding: {missing}"


def test_kernel_names_and_strerror(lib):
    lib.quota_kernel_name.restype = C.c_char_p
    lib.quota_strerror.restype = C.c_char_p
    from paper_2604_17320_amd import binding
    names = [lib.quota_kernel_name(i).decode() for i in range(binding.KERNEL_COUNT)]
    assert len(set(names)) == binding.KERNEL_COUNT and "?" not in names
    assert lib.quota_kernel_name(binding.KERNEL_COUNT).decode() == "?"
    assert lib.quota_kernel_name(-1).decode() == "?"
    msgs = [lib.quota_strerror(c).decode() for c in range(0, -6, -1)]
    assert len(set(msgs)) == 6                                 # distinct text per error code
    assert lib.quota_strerror(-99).decode() not in msgs


def test_null_and_shape_checks_come_before_device_work(lib):
    # every call below must be rejected on the host: there is no GPU in this process
    ERR_NULL = -1
    assert lib.quota_quantize_act(None, 4, 128, 128, None, None, None, None, None) == ERR_NULL
    assert lib.quota_w4a4_gemm(None, None, 4, None, None, 0, None, 0, None, None) == ERR_NULL
    assert lib.quota_topk_prune(None, 1, 8, 4, None, None) == ERR_NULL
    assert lib.quota_prefill_layer(None, None, 0, None, None, None, None, None) == ERR_NULL
    lib.quota_prefill_workspace_bytes.restype = C.c_size_t
    assert lib.quota_prefill_workspace_bytes(None, 1, 16) == 0
    lib.quota_attention_workspace_bytes.restype = C.c_size_t
    assert lib.quota_attention_workspace_bytes(1, 640, 32, 128) > 0


def test_recipe_matches_the_oracle():
    """Host-only entry points (Eq. 1-5): the library's recipe against the oracle's, on the CPU."""
    import numpy as np
    import oracle
    from paper_2604_17320_amd import binding, workloads as wl
    for seed, m, tau, p_min, V0 in [(0, 5, 1.0, 0.3, 576), (1, 12, 0.5, 0.1, 2880), (2, 1, 2.0, 0.5, 64),
                                    (3, 30, 0.2, 0.25, 576)]:
        S = wl.rng(seed, "S", m).lognormal(-3.0, 1.0, m)
        ref = oracle.recipe.make_recipe(S, tau, p_min, V0)
        got = binding.quota_make_recipe(S.tolist(), tau, p_min, V0)
        assert np.allclose(got["s_norm"], ref["s_norm"], rtol=0, atol=1e-14)
        assert np.allclose(got["pi"], ref["pi"], rtol=1e-13, atol=0)
        assert np.allclose(got["r"], ref["r"], rtol=0, atol=1e-14)
        for k_got, k_ref, r in zip(got["K"], ref["K"], ref["r"]):
            assert k_got == k_ref or abs(r * V0 - round(r * V0)) < 1e-6      # equal unless r V0 sits on an integer
        assert all(a >= b for a, b in zip(got["K"], got["K"][1:])) and got["K"][-1] >= int(np.ceil(p_min * V0 - 1e-9))
    sched = wl.schedule_for(wl.CONFIGS[2])
    assert binding.quota_gflops_ratio(sched, 576, 64, 4096, 11008) == pytest.approx(
        oracle.recipe.gflops_ratio(sched, 576, 64, 4096, 11008), rel=1e-13)
    assert binding.quota_gflops_ratio([576] * 4, 576, 64, 4096, 11008, 1e12, 1e9) == 100.0
    flat = binding.quota_make_recipe([0.2, 0.2, 0.2], 1.0, 0.3, 576)
    assert flat["s_norm"] == [0.5, 0.5, 0.5] and flat["K"][-1] == 173
    a = wl.rng(5, "n").uniform(0.1, 1, 8).tolist()
    b = wl.rng(6, "n").uniform(1, 2, 8).tolist()
    assert binding.quota_sensitivity(a, b, 1e-6) == pytest.approx(oracle.recipe.sensitivity(a, b, 1e-6), rel=1e-15)
    for bad in [dict(S=[0.1], tau=0.0, p_min=0.3, V0=10), dict(S=[float("nan")], tau=1.0, p_min=0.3, V0=10),
                dict(S=[0.1], tau=1.0, p_min=1.5, V0=10)]:
        with pytest.raises(binding.QuotaError) as e:
            binding.quota_make_recipe(**bad)
        assert e.value.code == binding.ERR_INVALID_ARG


def _fake_layer(binding, H=32, dh=128, F=11008, Hkv=0, null_weights=False):
    """A layer descriptor whose pointers are never dereferenced: every call below must be rejected by
    the host-side checks, before any device work."""
    d, hk = H * dh, (Hkv or H)
    P = 0 if null_weights else 0x1000
    W = lambda n, k: binding.Weights(n, k, P, P)
    return binding.Layer(H, dh, F, 1e-5, 0x1000, 0x1000, W(d + 2 * hk * dh, d), W(d, d), W(2 * F, d), W(d, F),
                         0x1000, 0x1000, 4096, Hkv)


def test_layer_calls_reject_every_downstream_limit_before_touching_anything(lib):
    """A layer call that returns an error has enqueued nothing and moved no descriptor: the limits of
    the later steps (row-kernel width, tokens the score kernel holds, rows the decode attention
    holds, cache capacity) are checked up front."""
    from paper_2604_17320_amd import binding
    ERR_NULL, ERR_INVALID, ERR_SHAPE, ERR_CAPACITY = -1, -2, -3, -4
    p = binding.ScoreParams(0.25, 0.45, 0.10, 0.20, 10, 90)

    def prefill(L, B, N, Nv, K, cache_len=0, capacity=100000, cache_ptr=0x1000, cacheH=None):
        cache = binding.KVCache(B, capacity, cacheH or (L.Hkv or L.H), L.dh, cache_len, cache_ptr, cache_ptr,
                                cache_ptr, cache_ptr)
        st = binding.State(B, N, 0, Nv, 0x1000, 0x1000, 0x1000, 0x1000)
        rc = lib.quota_prefill_layer(C.byref(L), C.byref(st), K, C.byref(p), C.byref(cache), None,
                                     C.c_void_p(0x1000), None)
        assert (cache.len, st.N, st.Nv) == (cache_len, N, Nv), "descriptors moved by a rejected call"
        return rc

    ok = _fake_layer(binding)
    assert prefill(_fake_layer(binding, F=32800), 1, 640, 576, 173) == ERR_SHAPE          # F > 32768
    assert prefill(_fake_layer(binding, F=11000), 1, 640, 576, 173) == ERR_SHAPE          # F % 32
    assert prefill(_fake_layer(binding, H=160), 1, 640, 576, 173) == ERR_SHAPE            # d = 20480 > 16384
    assert prefill(_fake_layer(binding, dh=96), 1, 640, 576, 173) == ERR_SHAPE
    assert prefill(_fake_layer(binding, Hkv=5), 1, 640, 576, 173) == ERR_SHAPE            # 32 % 5
    assert prefill(ok, 1, 8400, 8300, 500) == ERR_SHAPE                                   # 8300 scored tokens
    assert prefill(ok, 1, 640, 576, 173, cache_len=10, capacity=200) == ERR_CAPACITY      # 10 + 237 > 200
    assert prefill(ok, 1, 640, 576, 173, cache_len=-1) == ERR_INVALID
    assert prefill(ok, 1, 640, 576, -2) == ERR_INVALID
    assert prefill(ok, 1, 640, 700, 173) == ERR_INVALID                                   # Nv > N
    assert prefill(ok, 1, 640, 576, 173, cache_ptr=0) == ERR_NULL
    assert prefill(_fake_layer(binding, null_weights=True), 1, 640, 576, 173) == ERR_NULL
    assert prefill(ok, 1, 640, 576, 173, cacheH=8) == ERR_SHAPE                           # cache of another head count
    bad_w = _fake_layer(binding)
    bad_w.down = binding.Weights(4096, 11040, 0x1000, 0x1000)                             # K does not match F
    assert prefill(bad_w, 1, 640, 576, 173) == ERR_SHAPE
    # a layer outside the candidate set may carry any number of visual tokens (nothing is scored) -- the
    # only thing left to reject here is the capacity
    assert prefill(ok, 1, 8400, 8300, -1, capacity=100) == ERR_CAPACITY

    def decode(L, B, cache_len, capacity):
        cache = binding.KVCache(B, capacity, L.Hkv or L.H, L.dh, cache_len, 0x1000, 0x1000, 0x1000, 0x1000)
        rc = lib.quota_decode_layer(C.byref(L), C.c_void_p(0x1000), C.c_void_p(0x1000), B, C.byref(cache),
                                    C.c_void_p(0x1000), None, C.c_void_p(0x1000), None)
        assert cache.len == cache_len, "cache length moved by a rejected call"
        return rc

    assert decode(ok, 4, 300, 300) == ERR_CAPACITY
    assert decode(ok, 4, 8192, 9000) == ERR_SHAPE                                         # 8193 rows to attend over
    assert decode(_fake_layer(binding, F=32800), 4, 10, 100) == ERR_SHAPE
    assert decode(ok, 4, -3, 100) == ERR_INVALID


def test_gemm_variant_setter(lib):
    assert lib.quota_set_gemm_variant(5) == -2 and lib.quota_set_gemm_variant(-2) == -2
    for v in (0, 4, -1):
        assert lib.quota_set_gemm_variant(v) == 0


def test_profiler_calls_validate_before_any_device_work(lib):
    """The calibration-time entry points (Eq. 1) reject bad descriptors on the host: no GPU is needed
    to see the error codes, and the workspace queries answer 0 for a layer they would reject."""
    from paper_2604_17320_amd import binding as qb
    lib.quota_fp_block_workspace_bytes.restype = C.c_size_t
    lib.quota_profile_block_workspace_bytes.restype = C.c_size_t
    fake = 0x1000                                      # never dereferenced: every check below fails first
    good = qb.FpLayer(8, 64, 1376, 0, 1e-5, fake, fake, fake, fake, fake, fake, fake, fake, 64)
    assert lib.quota_fp_block_workspace_bytes(C.byref(good), 2, 80) > 0
    ws = C.c_void_p(fake)
    x = C.c_void_p(fake)
    assert lib.quota_fp_block(None, x, x, 2, 80, x, ws, None) == qb.ERR_NULL
    assert lib.quota_fp_block(C.byref(good), None, x, 2, 80, x, ws, None) == qb.ERR_NULL
    assert lib.quota_fp_block(C.byref(good), x, x, 0, 80, x, ws, None) == qb.ERR_INVALID_ARG
    for bad in (qb.FpLayer(8, 96, 1376, 0, 1e-5, fake, fake, fake, fake, fake, fake, fake, fake, 64),     # head size
                qb.FpLayer(8, 64, 1376, 3, 1e-5, fake, fake, fake, fake, fake, fake, fake, fake, 64),     # H % Hkv
                qb.FpLayer(8, 64, 1380, 0, 1e-5, fake, fake, fake, fake, fake, fake, fake, fake, 64)):    # F % 32
        assert lib.quota_fp_block(C.byref(bad), x, x, 2, 80, x, ws, None) == qb.ERR_SHAPE
        assert lib.quota_fp_block_workspace_bytes(C.byref(bad), 2, 80) == 0
    no_w = qb.FpLayer(8, 64, 1376, 0, 1e-5, fake, fake, None, fake, fake, fake, fake, fake, 64)
    assert lib.quota_fp_block(C.byref(no_w), x, x, 2, 80, x, ws, None) == qb.ERR_NULL
    assert lib.quota_activation_deviation(None, x, 2, C.c_long(10), x, x, None) == qb.ERR_NULL
    assert lib.quota_activation_deviation(x, x, 0, C.c_long(10), x, x, None) == qb.ERR_INVALID_ARG
    assert lib.quota_activation_deviation(x, x, 2, C.c_long(-1), x, x, None) == qb.ERR_INVALID_ARG
    # the two layers of a profile must describe the same block
    w = qb.Weights(64, 64, fake, fake)
    lq = qb.Layer(4, 64, 1376, 1e-5, fake, fake, w, w, w, w, fake, fake, 64, 0)
    cache = qb.KVCache(2, 100, 4, 64, 0, fake, fake, fake, fake)
    assert lib.quota_profile_block(C.byref(lq), C.byref(good), x, x, 2, 80, C.byref(cache), x, x, ws, None) == qb.ERR_SHAPE
    assert lib.quota_profile_block(C.byref(lq), C.byref(good), x, x, 2, 80, None, x, x, ws, None) == qb.ERR_NULL
    assert cache.len == 0
