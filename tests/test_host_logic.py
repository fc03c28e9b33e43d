"""CPU checks of the host-side helpers that hold no method arithmetic: the synthetic workload
definitions (shapes, the keep schedules the benchmark and the stack tests run) and the tool that
condenses profiler CSVs into the summaries under profiles/."""
import csv
import io
import json
import os
import subprocess
import sys

import numpy as np

from paper_2604_17320_amd import profile_summary as ps, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_config_shapes():
    c1, c2, c3 = wl.CONFIGS[0], wl.CONFIGS[1], wl.CONFIGS[2]
    assert (c1.d, c1.H, c1.dh, c1.F, c1.N) == (512, 8, 64, 1376, 80)
    for c in (c2, c3):
        assert (c.d, c.H, c.dh, c.F, c.Nv, c.Nt) == (4096, 32, 128, 11008, 576, 64)
    assert c3.layers == 32 and c3.B == 1


def test_stack_schedule_is_the_stated_ramp():
    """Full budget on the first two layers, then the linear ramp that ends at 0.1 and averages 0.30
    over the 32 layers; ceil of exact rationals."""
    K = wl.schedule_for(wl.CONFIGS[2])
    assert K[:6] == [576, 576, 235, 229, 223, 216] and K[-4:] == [76, 70, 64, 58] and len(K) == 32
    assert all(a >= b for a, b in zip(K, K[1:]))
    assert abs(sum(K) / (32 * 576) - 0.3008) < 2e-4
    assert wl.schedule_for(wl.CONFIGS[1]) == [173]              # ceil(0.3 * 576), Table 4's operating point


def test_generators_are_seeded_and_shaped():
    s = wl.CONFIGS[0]
    x = wl.hidden_state(s, 3)
    assert x.dtype == np.float16 and x.shape == (s.B * s.N, s.d)
    assert np.array_equal(x, wl.hidden_state(s, 3)) and not np.array_equal(x, wl.hidden_state(s, 4))
    col_rms = np.sqrt((x.astype(np.float32) ** 2).mean(axis=0))
    assert (col_rms > 10).sum() == s.n_outlier                  # the outlier channels, and only they
    cos, sin = wl.rope_tables(64, 16)
    assert cos.shape == (16, 32) and np.allclose(cos ** 2 + sin ** 2, 1.0, atol=1e-6) and np.all(cos[0] == 1.0)


def test_profile_summary_classifies_library_kernels():
    assert ps.classify("_ZN12_GLOBAL__N_116w4a4_gemm_kernelILi2ELi1ELi4ELi2ELb1ELb0ELb0ELi1EEEvPKh") == "w4a4_gemm_64x128"
    assert ps.classify("_ZN12_GLOBAL__N_116w4a4_gemm_kernelILi1ELi1ELi8ELi4ELb1ELb0ELb1ELi1EEEv") == "w4a4_gemm_32x128_deep"
    assert ps.classify("_Z27rmsnorm_quantize_act_kernelILb0ELi64ELi8EEv") == "rmsnorm_quantize_act"
    assert ps.classify("_Z19quantize_act_kernelILb1ELi64ELi8EEv") == "quantize_act"
    assert ps.bandwidth_case("_Z19quantize_act_kernelILb1ELi64ELi8EEv") == "quantize_act (+ m_mag, m_res)"
    assert ps.bandwidth_case("_Z27rmsnorm_quantize_act_kernelILb0ELi64ELi8EEv") == "rmsnorm_quantize_act"
    assert ps.classify("void at::native::elementwise_kernel<...>") is None


def test_profile_summary_stats_table(tmp_path, capsys):
    rows = [dict(Name="_Z19quantize_act_kernelILb0ELi64ELi8EEv", Calls=4, TotalDurationNs=100000),
            dict(Name="_ZN12_GLOBAL__N_115attn_fwd_kernelILi128EEEv", Calls=2, TotalDurationNs=30000),
            dict(Name="some_other_kernel", Calls=9, TotalDurationNs=999)]
    p = tmp_path / "stats.csv"
    with open(p, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=["Name", "Calls", "TotalDurationNs"])
        w.writeheader()
        w.writerows(rows)
    ps.stats(str(p))
    out = capsys.readouterr().out
    assert "quantize_act" in out and "25.00" in out and "attention_fwd" in out and "15.00" in out
    assert "some_other_kernel" not in out


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
