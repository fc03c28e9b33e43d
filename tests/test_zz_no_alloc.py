"""The entry point for callers that cannot allocate: quota_attention_prefill_static keeps its
intermediates in a device array inside the library instead of a caller workspace.  Its outputs
must equal those of quota_attention_prefill_gqa (same kernels, different scratch) bit for bit and
the oracle within the attention tolerances, on two calls in a row, the second one smaller (the
shared array then still holds the first call's values beyond the second call's extent)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17320_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _inputs(B, N, H, Hkv, dh, seed):
    r = wl.rng(seed, "noalloc", B, N, H)
    q = r.standard_normal((B * N, H * dh), dtype=np.float32).astype(np.float16)
    _, _, khat = oracle.kv_quant(r.standard_normal((B * N, Hkv * dh), dtype=np.float32).astype(np.float16))
    _, _, vhat = oracle.kv_quant(r.standard_normal((B * N, Hkv * dh), dtype=np.float32).astype(np.float16))
    return q, khat, vhat


def _close_f16(a, b, tol=1e-2):
    a, b = a.astype(np.float64), b.astype(np.float64)
    return np.all(np.abs(a - b) <= tol * np.maximum(np.abs(b), np.sqrt((b ** 2).mean())))


def test_static_scratch_attention_matches_workspace_attention():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_17320_amd import binding as qb
    qb.lib()
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for case, (B, N, H, Hkv, dh, vb, Nv) in enumerate([(2, 300, 8, 2, 128, 4, 250), (1, 90, 4, 4, 64, 0, 64)]):
        print(f"static-scratch attention case {case}: B={B} N={N} H={H} Hkv={Hkv} dh={dh}", flush=True)
        q, khat, vhat = _inputs(B, N, H, Hkv, dh, 900 + case)
        tq, tk, tv = dev(q), dev(khat), dev(vhat)
        outs = []
        for static in (False, True):
            o = torch.zeros((B * N, H * dh), dtype=torch.float16, device="cuda")
            ci = torch.zeros((B, Nv), dtype=torch.float32, device="cuda")
            cv = torch.zeros((B, Nv), dtype=torch.float32, device="cuda")
            if static:
                qb.quota_attention_prefill_static(tq, tk, tv, B, N, H, Hkv, dh, vb, Nv, o, ci, cv)
            else:
                ws = torch.empty(qb.quota_attention_workspace_bytes(B, N, H, dh), dtype=torch.uint8, device="cuda")
                qb.quota_attention_prefill_gqa(tq, tk, tv, B, N, H, Hkv, dh, vb, Nv, o, ci, cv, ws)
            torch.cuda.synchronize()
            outs.append((o.cpu().numpy(), ci.cpu().numpy(), cv.cpu().numpy()))
        (o_ws, ci_ws, cv_ws), (o_st, ci_st, cv_st) = outs
        assert np.array_equal(o_st.view(np.uint16), o_ws.view(np.uint16))
        assert np.array_equal(ci_st.view(np.uint32), ci_ws.view(np.uint32))
        assert np.array_equal(cv_st.view(np.uint32), cv_ws.view(np.uint32))
        o_ref, ci_ref, cv_ref = oracle.attention(q, khat, vhat, B, N, H, dh, vb, Nv, Hkv=Hkv)
        assert _close_f16(o_st, o_ref)
        assert np.allclose(ci_st, ci_ref, rtol=2e-5, atol=1e-7)
        assert np.allclose(cv_st, cv_ref, rtol=2e-5, atol=1e-7)


def test_static_scratch_attention_rejects_oversize():
    from paper_2604_17320_amd import binding as qb
    t = torch.zeros(8, dtype=torch.float16, device="cuda")
    f = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(qb.QuotaError) as e:          # 4 * 64 * 1025 rows > 262144: rejected on the host
        qb.quota_attention_prefill_static(t, t, t, 4, 1025, 64, 64, 128, 0, 8, t, f, f)
    assert e.value.code == qb.ERR_CAPACITY
