"""GPU parity at the full sizes of the batched-serving shape (7B, batch 16, 576 + 128 tokens) and the
high-resolution 13B shape (d=5120, 40 heads, FFN 13824, 2880 + 64 tokens).  The oracle cannot run
these whole in reasonable time, so every kernel runs at full size on the GPU and is compared on
SAMPLED rows / heads / sequences that the oracle computes one by one (all these operations are
independent per row, per head or per sequence, so a sample is checked to the same bar as a full
comparison: bit-exact for codes, scales and GEMM outputs, tolerance for attention)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl
from test_gpu_ops import _act, _pack4, close_f16, dev, host, unpack4
from test_gpu_layer import build_layer, check_free_running, run_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available()
    from paper_2604_17320_amd import binding
    binding.lib()
    return binding


def sample_rows(M, n, seed):
    edge = [0, 1, 31, 32, 63, 64, 127, 128, M - 129, M - 65, M - 64, M - 33, M - 2, M - 1]
    r = wl.rng(seed, "rows", M)
    rows = sorted(set(int(v) for v in edge if 0 <= v < M) | set(r.integers(0, M, n).tolist()))
    return np.array(rows, np.int64)


@pytest.mark.parametrize("M,d", [(11264, 4096), (11776, 5120)])
def test_quantizers_full_size_sampled_rows(qb, M, d):
    x = _act(M, d, 81, 1.3)
    gamma = wl.rng(81, "gamma", d).uniform(0.5, 1.5, d).astype(np.float32)
    rows = sample_rows(M, 200, 81)
    xd = dev(x)
    qp = torch.empty((M, d // 2), dtype=torch.uint8, device="cuda")
    sc, sq, rq = (torch.empty(M, dtype=torch.float32, device="cuda") for _ in range(3))
    qb.quota_quantize_act(xd, M, d, d, qp, sc, sq, rq)
    q, s, ss, rs = oracle.quantize_act(x[rows])
    assert np.array_equal(unpack4(host(qp)[rows]), q) and np.array_equal(host(sc)[rows], s)
    assert np.array_equal(host(sq)[rows], ss) and np.array_equal(host(rq)[rows], rs)
    h = torch.empty((M, d), dtype=torch.float16, device="cuda")
    qb.quota_rmsnorm_quantize_act(xd, M, d, d, dev(gamma), 1e-5, qp, sc, sq, rq, h)
    h_ref = oracle.rmsnorm(x[rows], gamma, 1e-5)
    q, s, _, _ = oracle.quantize_act(h_ref)
    assert np.array_equal(host(h)[rows].view(np.uint16), h_ref.view(np.uint16))
    assert np.array_equal(unpack4(host(qp)[rows]), q) and np.array_equal(host(sc)[rows], s)
    assert np.array_equal(host(sq)[rows], ss)           # side outputs describe the layer input, not h


def test_silu_mul_quantize_13b_ffn_sampled_rows(qb):
    M, F = 2944, 13824
    gu = _act(M, 2 * F, 82, 1.5)
    rows = sample_rows(M, 40, 82)
    qp = torch.empty((M, F // 2), dtype=torch.uint8, device="cuda")
    sc = torch.empty(M, dtype=torch.float32, device="cuda")
    z_ref = oracle.silu_mul(gu[rows], F)
    zin = np.zeros((M, F), np.float16)
    zin[rows] = z_ref
    qb.quota_silu_mul_quantize_act(dev(gu), M, F, qp, sc, None, dev(zin))     # teacher-forced product
    q, s, _, _ = oracle.quantize_act(z_ref)
    assert np.array_equal(unpack4(host(qp)[rows]), q) and np.array_equal(host(sc)[rows], s)
    z = torch.empty((M, F), dtype=torch.float16, device="cuda")
    qb.quota_silu_mul_quantize_act(dev(gu), M, F, qp, sc, z, None)            # the library's own product
    assert close_f16(host(z)[rows], z_ref, tol=2e-3)


@pytest.mark.parametrize("M,N,K,nrows", [(11264, 12288, 4096, 40),     # batch-16 QKV
                                         (11264, 4096, 11008, 40),     # batch-16 down projection
                                         (2944, 27648, 5120, 16),      # 13B gate/up, one sequence
                                         (11776, 5120, 13824, 24)])    # 13B down projection, batch 4
def test_w4a4_gemm_full_size_sampled_rows(qb, M, N, K, nrows):
    from paper_2604_17320_amd.model import PackedLinear
    r = wl.rng(83, "gemm-full", M, N, K)
    w = r.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    qw, sw = oracle.quantize_weights(w)
    del w
    qa = r.integers(-8, 8, (M, K), dtype=np.int8)
    sa = r.uniform(0.01, 2.0, M).astype(np.float32)
    rows = sample_rows(M, nrows, 83)
    res = r.standard_normal((M, N), dtype=np.float32).astype(np.float16)
    lin = PackedLinear.from_codes(dev(qw), dev(sw))
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    qb.quota_w4a4_gemm(dev(_pack4(qa)), dev(sa), M, lin.desc, y, N, dev(res), N)
    y_ref = oracle.w4a4_gemm(qa[rows], sa[rows], qw, sw, residual=res[rows])
    assert np.array_equal(host(y)[rows].view(np.uint16), y_ref.view(np.uint16))


def test_rope_kv_quant_full_size_sampled_rows(qb):
    H, dh, M = 40, 128, 11776
    d = H * dh
    qkv = _act(M, 3 * d, 84, 2.0)
    pos = (np.arange(M, dtype=np.int32) % 2944).astype(np.int32)
    cos, sin = wl.rope_tables(dh, 2944)
    rows = sample_rows(M, 60, 84)
    t16 = lambda: torch.empty((M, d), dtype=torch.float16, device="cuda")
    q_rot, khat, vhat = t16(), t16(), t16()
    kc, vc = (torch.empty((M, d // 2), dtype=torch.uint8, device="cuda") for _ in range(2))
    ks, vs = (torch.empty((M, d // 64), dtype=torch.float16, device="cuda") for _ in range(2))
    qb.quota_rope_kv_quant(dev(qkv), M, H, dh, dev(pos), dev(cos), dev(sin), 2944, q_rot, khat, vhat, kc, ks, vc, vs)
    s = qkv[rows]
    q_ref = oracle.rope(s[:, :d], H, dh, pos[rows], cos, sin)
    k_ref = oracle.rope(s[:, d:2 * d], H, dh, pos[rows], cos, sin)
    kc_ref, ks_ref, kh_ref = oracle.kv_quant(k_ref)
    vc_ref, vs_ref, vh_ref = oracle.kv_quant(np.ascontiguousarray(s[:, 2 * d:]))
    eq = lambda a, b: np.array_equal(np.ascontiguousarray(a).view(np.uint16), b.view(np.uint16))
    assert eq(host(q_rot)[rows], q_ref) and eq(host(khat)[rows], kh_ref) and eq(host(vhat)[rows], vh_ref)
    assert np.array_equal(unpack4(host(kc)[rows]), kc_ref) and np.array_equal(unpack4(host(vc)[rows]), vc_ref)
    assert eq(host(ks)[rows], ks_ref) and eq(host(vs)[rows], vs_ref)


def test_attention_high_resolution_length(qb):
    """2880 visual + 64 text tokens: 46 query tiles, a ragged last key tile; two heads are enough for
    the oracle, the per-head work is what scales with the sequence."""
    B, N, H, dh, vb, Nv = 1, 2944, 2, 128, 0, 2880
    d = H * dh
    q = _act(B * N, d, 85, 1.0)
    _, _, khat = oracle.kv_quant(_act(B * N, d, 86, 1.0))
    _, _, vhat = oracle.kv_quant(_act(B * N, d, 87, 1.0))
    o_ref, ci_ref, cv_ref = oracle.attention(q, khat, vhat, B, N, H, dh, vb, Nv)
    o = torch.empty((B * N, d), dtype=torch.float16, device="cuda")
    ci, cv = (torch.zeros((B, Nv), dtype=torch.float32, device="cuda") for _ in range(2))
    ws = torch.empty(qb.quota_attention_workspace_bytes(B, N, H, dh), dtype=torch.uint8, device="cuda")
    qb.quota_attention_prefill(dev(q), dev(khat), dev(vhat), B, N, H, dh, vb, Nv, o, ci, cv, ws)
    assert close_f16(host(o), o_ref)
    assert np.allclose(host(ci), ci_ref, rtol=5e-5, atol=1e-7)
    assert np.allclose(host(cv), cv_ref, rtol=5e-5, atol=1e-7)
    # every query row's probabilities sum to 1, so all column masses (visual + text keys) sum to N
    # per head; the visual part alone is what the cues cover: check it against the oracle's total
    assert abs(float(host(ci).sum() + host(cv).sum()) - float(ci_ref.sum() + cv_ref.sum())) < 1e-2


def test_layer_batched_serving_shape_sampled_sequence(qb):
    """The 7B layer at batch 16 x (576 + 128) tokens, keep 173, free-running on the GPU; one sampled
    sequence is compared with the oracle run on that sequence alone (sequences do not interact)."""
    base = wl.CONFIGS[1]
    shape = wl.Shape("c4_layer", d=base.d, H=base.H, F=base.F, layers=1, B=16, Nv=576, Nt=128,
                     n_outlier=base.n_outlier, vis_begin=0)
    W, L, cos, sin = build_layer(shape, 0)
    x, pos = wl.hidden_state(shape, 4), wl.positions(shape)
    K, b = 173, 11
    got = run_gpu(qb, L, shape, x, pos, K)
    N, n_keep = shape.N, shape.N - shape.Nv + K
    one = wl.Shape("c4_one", d=base.d, H=base.H, F=base.F, layers=1, B=1, Nv=576, Nt=128,
                   n_outlier=base.n_outlier, vis_begin=0)
    xb = x.reshape(16, N, -1)[b]
    pb = pos.reshape(16, N)[b]
    ref = oracle.prefill_layer(W, xb, pb, 1, N, 0, 576, K, cos, sin, prune_mid=True)
    rows_all = slice(b * N, (b + 1) * N)
    rows_keep = slice(b * n_keep, (b + 1) * n_keep)
    sub = dict(qkv=got["qkv"][rows_all], o=got["o"][rows_all], score=got["score"][b:b + 1],
               keep_idx=got["keep_idx"][b:b + 1], rows=got["rows"][b:b + 1],
               cache_kc=got["cache_kc"][rows_keep], cache_vc=got["cache_vc"][rows_keep],
               x1=got["x1"][rows_keep], gu=got["gu"][rows_keep], z=got["z"][rows_keep],
               x_next=got["x_next"][rows_keep], pos_next=got["pos_next"][rows_keep])
    check_free_running(ref, sub, one, K, W)
    assert got["N"] == n_keep and got["Nv"] == K and got["cache_len"] == n_keep
    # every sequence keeps exactly K visual tokens, ascending, and all text tokens
    for bb in range(16):
        idx = got["keep_idx"][bb, :K]
        assert np.all(np.diff(idx) > 0) and idx.min() >= 0 and idx.max() < 576
        assert np.array_equal(got["rows"][bb, K:], np.arange(576, N))


def test_layer_13b_high_resolution_shape(qb):
    """One whole layer of the high-resolution 13B shape (d=5120, 40 heads, FFN 13824, 2880 visual + 64
    text tokens, budget 766 = the schedule's first pruning layer), one sequence: teacher-forced
    bit-exact and free-running within tolerance.  The largest N_v, N and FFN width the kernels meet."""
    from test_gpu_layer import assert_teacher_forced_exact
    shape = wl.Shape("c5_layer", d=5120, H=40, F=13824, layers=1, B=1, Nv=2880, Nt=64, n_outlier=51, vis_begin=0)
    W, L, cos, sin = build_layer(shape, 0)
    x, pos = wl.hidden_state(shape, 5), wl.positions(shape)
    K = 766
    ref = oracle.prefill_layer(W, x, pos, 1, shape.N, 0, shape.Nv, K, cos, sin, prune_mid=True)
    got = run_gpu(qb, L, shape, x, pos, K, dict(o=ref["o"], z=ref["z"], cm_inter=ref["cm_inter"],
                                                cm_intra=ref["cm_intra"]))
    assert_teacher_forced_exact(ref, got, shape, K)
    free = run_gpu(qb, L, shape, x, pos, K)
    check_free_running(ref, free, shape, K, W)


def test_layer_serving_shape_batch16(qb):
    """One whole layer at the batched-serving shape (batch 16 x (576 + 128) tokens of the 7B model,
    budget 235 as at layer 2 of the stack schedule): 11264 rows through the QKV projection and
    attention, 16 x 363 kept rows through the rest, teacher-forced bit-exact against the oracle,
    then one decode step of the 16 sequences over the pruned cache."""
    from test_gpu_layer import build_layer, run_gpu, assert_teacher_forced_exact
    from test_gpu_decode import check_decode
    base = wl.CONFIGS[1]
    shape = wl.Shape("c4_layer", d=base.d, H=base.H, F=base.F, layers=1, B=16, Nv=576, Nt=128,
                     n_outlier=base.n_outlier, vis_begin=0)
    K = 235
    W, L, cos, sin = build_layer(shape, 4)
    x, pos = wl.hidden_state(shape, 4), wl.positions(shape)
    ref = oracle.prefill_layer(W, x, pos, shape.B, shape.N, 0, shape.Nv, K, cos, sin, prune_mid=True)
    got = run_gpu(qb, L, shape, x, pos, K, dict(o=ref["o"], z=ref["z"], cm_inter=ref["cm_inter"],
                                                cm_intra=ref["cm_intra"]))
    assert_teacher_forced_exact(ref, got, shape, K)
    check_decode(qb, shape, 4, K, steps=1)
