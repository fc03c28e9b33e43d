"""GPU parity of a whole layer stack: the compacted hidden state, positions and per-layer 4-bit KV
caches carried from layer to layer through prefill, then decode steps that read those caches.
Teacher-forced per layer (oracle attention output, cues and SwiGLU product injected), so every
integer and fp16 tensor that crosses a layer boundary must be bit-exact; plus a HIP-graph replay
check of the same stack."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl
from test_gpu_ops import dev, host, unpack4
from test_gpu_layer import build_layer
from test_gpu_decode import eq16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available()
    from paper_2604_17320_amd import binding
    binding.lib()
    return binding


def small_stack(n_layers, B, budgets, decode_capacity=0, Hkv=None):
    from paper_2604_17320_amd.model import PrefillStack
    base = wl.CONFIGS[0]
    shape = wl.Shape("stack", d=base.d, H=base.H, F=base.F, layers=n_layers, B=B, Nv=base.Nv, Nt=base.Nt,
                     n_outlier=base.n_outlier, vis_begin=0)
    Ws, Ls = [], []
    for l in range(n_layers):
        if Hkv is None:
            W, L, cos, sin = build_layer(shape, 10 + l, gamma_random=True)
        else:                                   # grouped K/V heads
            from test_gpu_gqa import build_gqa_layer
            W, L, cos, sin = build_gqa_layer(shape.d, shape.H, Hkv, shape.dh, shape.F, 10 + l, shape.N + 8)
        Ws.append(W)
        Ls.append(L)
    stack = PrefillStack(Ls, B, shape.N, 0, shape.Nv, budgets, decode_capacity=decode_capacity)
    return shape, Ws, stack, cos, sin


def oracle_prefill(shape, Ws, budgets, x, pos, cos, sin):
    outs, N, Nv = [], shape.N, shape.Nv
    for W, K in zip(Ws, budgets):
        o = oracle.prefill_layer(W, x, pos, shape.B, N, 0, Nv, K, cos, sin, prune_mid=True)
        outs.append(o)
        x, pos, N, Nv = o["x_next"], o["pos_next"], o["n_keep"], o["Nv_next"]
    return outs


def test_stack_prefill_then_decode_teacher_forced(qb):
    from paper_2604_17320_amd.model import make_taps
    budgets = [64, 40, 19, 10]
    B = 2
    shape, Ws, stack, cos, sin = small_stack(4, B, budgets, decode_capacity=4)
    x, pos = wl.hidden_state(shape, 3), wl.positions(shape)
    ref = oracle_prefill(shape, Ws, budgets, x, pos, cos, sin)
    keep = []
    taps = []
    for o in ref:
        t = {k: dev(o[k]) for k in ("o", "z", "cm_inter", "cm_intra")}
        keep.append(t)
        taps.append(make_taps(inject_o=t["o"], inject_z=t["z"], inject_cm_inter=t["cm_inter"],
                              inject_cm_intra=t["cm_intra"]))
    xo, po, N, Nv = stack.run(dev(x), dev(pos), taps)
    last = ref[-1]
    assert (N, Nv) == (last["n_keep"], last["Nv_next"]) == (10 + shape.Nt, 10)
    assert eq16(host(xo), last["x_next"]) and np.array_equal(host(po), last["pos_next"])
    for l, o in enumerate(ref):
        c, n = stack.caches[l], o["n_keep"]
        assert c.len == n
        assert np.array_equal(unpack4(host(c.k_codes)[:, :n]).reshape(B * n, -1), o["cache_kc"])
        assert np.array_equal(unpack4(host(c.v_codes)[:, :n]).reshape(B * n, -1), o["cache_vc"])
        assert eq16(host(c.k_scales)[:, :n].reshape(B * n, -1), o["cache_ks"])
        assert eq16(host(c.v_scales)[:, :n].reshape(B * n, -1), o["cache_vs"])

    # decode: every layer appends to and reads its own pruned cache
    caches = [oracle.cache_from_prefill(o, B) for o in ref]
    r = wl.rng(3, "stack-decode")
    for step in range(3):
        xn = r.standard_normal((B, shape.d)).astype(np.float16)
        pn = np.full(B, shape.N + step, np.int32)
        xin, drefs = xn, []
        for l, W in enumerate(Ws):
            d_ = oracle.decode_layer(W, xin, pn, caches[l], cos, sin)
            drefs.append(d_)
            caches[l] = d_["cache"]
            xin = d_["x_next"]
        dk = [{k: dev(d_[k]) for k in ("o", "z")} for d_ in drefs]
        dt = [make_taps(inject_o=t["o"], inject_z=t["z"]) for t in dk]
        got = stack.decode(dev(xn), dev(pn), dt)
        assert eq16(host(got), drefs[-1]["x_next"])
        for l in range(len(Ws)):
            n = caches[l]["kc"].shape[1]
            assert stack.caches[l].len == n
            assert np.array_equal(unpack4(host(stack.caches[l].k_codes)[:, :n]), caches[l]["kc"])
            assert eq16(host(stack.caches[l].v_scales)[:, :n], caches[l]["vs"])


def test_stack_hip_graph_replays_equal_eager(qb):
    """The benchmark times a HIP graph of the stack: every replay must reproduce the eager result."""
    budgets = [64, 30, 12]
    shape, Ws, stack, cos, sin = small_stack(3, 1, budgets)
    x, pos = dev(wl.hidden_state(shape, 5)), dev(wl.positions(shape))
    xo, po, N, Nv = stack.run(x, pos)
    torch.cuda.synchronize()
    want_x, want_p = xo.clone(), po.clone()
    want_c = [c.k_codes.clone() for c in stack.caches]
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        stack.run(x, pos)                 # warm-up on the capture stream
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        gx, gp, _, _ = stack.run(x, pos)
    for rep in range(3):
        gx.zero_()
        for c in stack.caches:
            c.k_codes.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(gx, want_x) and torch.equal(gp, want_p), rep
        for c, w in zip(stack.caches, want_c):
            n = c.len
            assert torch.equal(c.k_codes[:, :n], w[:, :n]), rep
        stack.run(x, pos)                 # eager work between replays
        torch.cuda.synchronize()


def test_stack_prunes_at_candidate_layers_only(qb):
    """The recipe prunes at the candidate layers only: layers marked KEEP_ALL run no cue pass, no
    score and no top-k and keep every token.  For the oracle such a layer is one whose budget keeps
    everything (its scores then change nothing).  Six layers, candidates 2..3; teacher-forced, so the
    hidden state, positions and every layer's 4-bit cache must be bit-exact."""
    from paper_2604_17320_amd.model import make_taps
    budgets = [qb.KEEP_ALL, qb.KEEP_ALL, 30, 12, qb.KEEP_ALL, qb.KEEP_ALL]
    oracle_budgets = [10 ** 6, 10 ** 6, 30, 12, 10 ** 6, 10 ** 6]
    B = 2
    shape, Ws, stack, cos, sin = small_stack(6, B, budgets)
    x, pos = wl.hidden_state(shape, 9), wl.positions(shape)
    ref = oracle_prefill(shape, Ws, oracle_budgets, x, pos, cos, sin)
    keep, taps = [], []
    score_taps = []
    for l, o in enumerate(ref):
        t = {k: dev(o[k]) for k in ("o", "z", "cm_inter", "cm_intra")}
        sc = torch.full((B, o["score"].shape[1]), -7.0, dtype=torch.float32, device="cuda")
        keep.append(t)
        score_taps.append(sc)
        taps.append(make_taps(inject_o=t["o"], inject_z=t["z"], inject_cm_inter=t["cm_inter"],
                              inject_cm_intra=t["cm_intra"], score=sc))
    xo, po, N, Nv = stack.run(dev(x), dev(pos), taps)
    last = ref[-1]
    assert (N, Nv) == (last["n_keep"], last["Nv_next"]) == (12 + shape.Nt, 12)
    assert eq16(host(xo), last["x_next"]) and np.array_equal(host(po), last["pos_next"])
    for l, o in enumerate(ref):
        c, n = stack.caches[l], o["n_keep"]
        assert c.len == n
        assert np.array_equal(unpack4(host(c.k_codes)[:, :n]).reshape(B * n, -1), o["cache_kc"])
        assert eq16(host(c.v_scales)[:, :n].reshape(B * n, -1), o["cache_vs"])
        # a layer outside the candidate set produced no score at all; a candidate layer produced the oracle's
        got_sc = host(score_taps[l])
        if budgets[l] == qb.KEEP_ALL:
            assert np.all(got_sc == -7.0)
        else:
            assert np.array_equal(got_sc, o["score"])


@pytest.mark.parametrize("Hkv", [None, 2])
def test_stack_decode_loop_in_a_hip_graph(qb, Hkv):
    """A decode loop captured once and replayed: the cache length lives on the device (step count read
    by the kernels), the new token's input and position are refreshed in place between replays.
    Every replay must give the bits of the eager step with host-side lengths, appended rows included.
    Once with a K/V head per query head, once with grouped K/V heads (8 query heads on 2)."""
    budgets = [64, 30, 12]
    B, steps = 2, 4
    shape, Ws, stack, cos, sin = small_stack(3, B, budgets, decode_capacity=steps + 1, Hkv=Hkv)
    x, pos = dev(wl.hidden_state(shape, 6)), dev(wl.positions(shape))
    stack.run(x, pos)
    torch.cuda.synchronize()
    base_len = [c.len for c in stack.caches]
    r = wl.rng(6, "graph-decode")
    xs = [dev(r.standard_normal((B, shape.d)).astype(np.float16)) for _ in range(steps)]
    # eager reference with host-side lengths
    want = []
    for i in range(steps):
        pn = torch.full((B,), shape.N + i, dtype=torch.int32, device="cuda")
        want.append(stack.decode(xs[i], pn).clone())
    torch.cuda.synchronize()
    want_k = [c.k_codes.clone() for c in stack.caches]
    want_s = [c.v_scales.clone() for c in stack.caches]
    # rewind, clear the appended rows, and run the same steps as replays of one captured step
    for c, n in zip(stack.caches, base_len):
        c.desc.len = n
        c.k_codes[:, n:].zero_()
        c.v_scales[:, n:].zero_()
    step_dev = stack.begin_stepped_decode(steps)
    x_in = torch.zeros((B, shape.d), dtype=torch.float16, device="cuda")
    pn = torch.full((B,), shape.N, dtype=torch.int32, device="cuda")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        stack.decode(x_in, pn)                     # warm-up on the capture stream (writes row base_len: rewritten below)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        y = stack.decode(x_in, pn)
        qb.quota_advance_step(step_dev)
        pn.add_(1)
    step_dev.zero_()
    pn.fill_(shape.N)
    for i in range(steps):
        x_in.copy_(xs[i])
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want[i]), i
        assert int(step_dev.item()) == i + 1
    stack.end_stepped_decode(steps)
    for c, n, wk, ws_ in zip(stack.caches, base_len, want_k, want_s):
        assert c.len == n + steps
        assert torch.equal(c.k_codes[:, : n + steps], wk[:, : n + steps])
        assert torch.equal(c.v_scales[:, : n + steps], ws_[:, : n + steps])
