"""The headline configuration at its full depth: the 32-layer 7B-shaped W4A4 pruned prefill
(576 visual + 64 text tokens, the benchmark's budget schedule 576, 576, 235, ... , 58, the benchmark's
own seeded weights), layer by layer against the oracle with the weights streamed one layer at a time.
Teacher-forced (the oracle's attention output, cues and SwiGLU product injected), so the hidden
state, positions, kept index sets and each layer's 4-bit cache must be bit-exact through all 32
layers.  Split into four runs of eight layers that continue each other, so that no single test
stays silent for long."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl
from test_gpu_ops import dev, host, unpack4

pytestmark = pytest.mark.gpu

SHAPE = wl.CONFIGS[2]
STATE = {}


def _layer(qb, l, cos, sin, cosT, sinT):
    """Layer l of the benchmark's stack: weights from the benchmark's device generator, quantized by the
    ORACLE for both sides (and once more by the library, which must agree code for code)."""
    from paper_2604_17320_amd.model import PackedLinear, PrefillLayer
    fw = wl.fp_weights_device(SHAPE, 0, l)
    q, lin = {}, {}
    for name, w in fw.items():
        codes, scales = oracle.quantize_weights(w.cpu().numpy())
        q[name] = (codes, scales)
        lin[name] = PackedLinear.from_codes(dev(codes), dev(scales))
        if name == "o":                                  # the benchmark quantizes on the GPU: same codes
            own = PackedLinear.from_fp32(w, keep_plain=True)
            assert torch.equal(own.packed, lin[name].packed) and torch.equal(own.scales, lin[name].scales)
            del own
    del fw
    g = np.ones(SHAPE.d, np.float32)
    W = oracle.LayerWeights(qkv=q["qkv"], o=q["o"], gu=q["gu"], down=q["down"], gamma1=g, gamma2=g, eps=1e-5,
                            H=SHAPE.H, dh=SHAPE.dh, F=SHAPE.F)
    gd = torch.ones(SHAPE.d, dtype=torch.float32, device="cuda")
    L = PrefillLayer(SHAPE.H, SHAPE.dh, SHAPE.F, lin["qkv"], lin["o"], lin["gu"], lin["down"], gd, gd, 1e-5, cosT, sinT)
    return W, L


@pytest.mark.parametrize("first", [0, 8, 16, 24])
def test_c3_stack_full_depth_teacher_forced(first):
    assert torch.cuda.is_available()
    from paper_2604_17320_amd import binding as qb
    from paper_2604_17320_amd.model import KVCache4, make_taps
    budgets = wl.schedule_for(SHAPE)
    assert len(budgets) == 32 and budgets[:3] == [576, 576, 235] and budgets[-1] == 58
    if first == 0:
        STATE.clear()
        STATE.update(x=wl.hidden_state(SHAPE, 0), pos=wl.positions(SHAPE), N=SHAPE.N, Nv=SHAPE.Nv)
    assert STATE.get("next", 0) == first, "the four parts run in order"
    cos, sin = wl.rope_tables(SHAPE.dh, SHAPE.N)
    cosT, sinT = dev(cos), dev(sin)
    d = SHAPE.d
    for l in range(first, first + 8):
        K, N, Nv = budgets[l], STATE["N"], STATE["Nv"]
        W, L = _layer(qb, l, cos, sin, cosT, sinT)
        ref = oracle.prefill_layer(W, STATE["x"], STATE["pos"], 1, N, 0, Nv, K, cos, sin, prune_mid=True)
        n_keep, k = ref["n_keep"], ref["Nv_next"]
        inj = {n_: dev(ref[n_]) for n_ in ("o", "z", "cm_inter", "cm_intra")}
        keep_idx = torch.zeros((1, k), dtype=torch.int32, device="cuda")
        score = torch.zeros((1, Nv), dtype=torch.float32, device="cuda")
        taps = make_taps(inject_o=inj["o"], inject_z=inj["z"], inject_cm_inter=inj["cm_inter"],
                         inject_cm_intra=inj["cm_intra"], keep_idx=keep_idx, score=score)
        cache = KVCache4(1, n_keep, SHAPE.H, SHAPE.dh)
        x_out = torch.zeros((n_keep, d), dtype=torch.float16, device="cuda")
        pos_out = torch.zeros((n_keep,), dtype=torch.int32, device="cuda")
        ws = torch.empty(L.workspace_bytes(1, N), dtype=torch.uint8, device="cuda")
        xd, pd = dev(STATE["x"]), dev(STATE["pos"])
        st = qb.State(1, N, 0, Nv, xd.data_ptr(), pd.data_ptr(), x_out.data_ptr(), pos_out.data_ptr())
        qb.quota_prefill_layer(L.desc, st, K, qb.quota_score_params_default(), cache.desc, taps, ws)
        where = f"layer {l}"
        assert (st.N, st.Nv, cache.len) == (n_keep, k, n_keep), where
        assert np.array_equal(host(score), ref["score"]), where
        assert np.array_equal(host(keep_idx), ref["keep_idx"]), where
        assert np.array_equal(host(pos_out), ref["pos_next"]), where
        assert np.array_equal(host(x_out).view(np.uint16), ref["x_next"].view(np.uint16)), where
        assert np.array_equal(unpack4(host(cache.k_codes)[0]), ref["cache_kc"]), where
        assert np.array_equal(unpack4(host(cache.v_codes)[0]), ref["cache_vc"]), where
        assert np.array_equal(host(cache.k_scales)[0].view(np.uint16), ref["cache_ks"].view(np.uint16)), where
        assert np.array_equal(host(cache.v_scales)[0].view(np.uint16), ref["cache_vs"].view(np.uint16)), where
        STATE.update(x=ref["x_next"], pos=ref["pos_next"], N=n_keep, Nv=k, next=l + 1)
        del W, L, cache, ws, inj
    if first == 24:
        assert (STATE["N"], STATE["Nv"]) == (58 + 64, 58)
