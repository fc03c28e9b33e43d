#!/usr/bin/env python3
"""Benchmark of the QUOTA hot path on one MI355X.

One "step" = one prefill pass of the whole layer stack (every kernel of the
path, all layers) over one batch of seeded synthetic input.  Prints ONE JSON
line: prefill tokens/s, the roofline figure of the dominant kernel, per-kernel
timings, and the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3|c2|c1]
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, TOP/s
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, GB/s


def build_stack(shape, seed, budgets, keep_plain_layers=()):
    import torch
    from paper_2604_17320_amd import workloads as wl
    from paper_2604_17320_amd.model import PackedLinear, PrefillLayer, PrefillStack
    d, F = shape.d, shape.F
    cos, sin = wl.rope_tables(shape.dh, shape.N)
    cosT, sinT = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    gamma = torch.ones(d, dtype=torch.float32, device="cuda")
    layers = []
    for l in range(shape.layers):
        g = torch.Generator(device="cuda")
        g.manual_seed(seed * 1000 + l)
        lin = {}
        for name, (n, k) in dict(qkv=(3 * d, d), o=(d, d), gu=(2 * F, d), down=(d, F)).items():
            w = torch.randn((n, k), generator=g, device="cuda", dtype=torch.float32) * 0.02
            lin[name] = PackedLinear.from_fp32(w, keep_plain=l in keep_plain_layers)
            del w
        layers.append(PrefillLayer(shape.H, shape.dh, F, lin["qkv"], lin["o"], lin["gu"], lin["down"],
                                   gamma, gamma, 1e-5, cosT, sinT))
    torch.cuda.synchronize()
    stack = PrefillStack(layers, shape.B, shape.N, shape.vis_begin, shape.Nv, budgets)
    return stack, (cos, sin)


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed counter profile (two rocprofv3 --pmc
    passes, FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_c3_stack.txt")
    try:
        with open(path) as f:
            rec = json.load(f)["kernels"].get(kernel)
    except (OSError, ValueError, KeyError):
        return None
    return rec and dict(bytes_per_launch=rec["fetch_bytes"] + rec["write_bytes"], fetch_bytes=rec["fetch_bytes"],
                        write_bytes=rec["write_bytes"], algorithmic_bytes=rec.get("algorithmic_bytes"),
                        source="profiles/hbm_traffic_c3_stack.txt")


def serving_shape_kernels(shape, seed, reps=20):
    """The same kernels at the batched-serving shape (batch 16 x 704 tokens of the 7B model), where a
    call moves >= 90 MB and the bandwidth kernels are out of the launch-latency regime: each kernel is
    launched `reps` times back to back between one event pair, and its algorithmic bytes (or ops) per
    second are set against the HBM (or int8 MFMA) peak.  Supplementary to the headline figure."""
    import torch
    from paper_2604_17320_amd import binding as qb, workloads as wl
    from paper_2604_17320_amd.model import KVCache4, PackedLinear
    B, N, d, H, dh, F = 16, 704, shape.d, shape.H, shape.dh, shape.F
    M = B * N
    g = torch.Generator(device="cuda")
    g.manual_seed(seed + 77)
    rnd = lambda *shp: torch.randn(shp, generator=g, device="cuda", dtype=torch.float32).to(torch.float16)
    x, qkv, gu = rnd(M, d), rnd(M, 3 * d), rnd(M, 2 * F)
    gamma = torch.ones(d, dtype=torch.float32, device="cuda")
    qa = torch.empty((M, max(d, F) // 2), dtype=torch.uint8, device="cuda")
    sa, sq, rq = (torch.empty(M, dtype=torch.float32, device="cuda") for _ in range(3))
    cos, sin = wl.rope_tables(dh, N)
    cosT, sinT = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    pos = torch.arange(N, dtype=torch.int32, device="cuda").repeat(B)
    q_rot, khat, vhat = (torch.empty((M, d), dtype=torch.float16, device="cuda") for _ in range(3))
    kc, vc = (torch.empty((M, d // 2), dtype=torch.uint8, device="cuda") for _ in range(2))
    ks, vs = (torch.empty((M, d // 64), dtype=torch.float16, device="cuda") for _ in range(2))
    n_keep = 173 + 128
    keep = torch.arange(n_keep, dtype=torch.int32, device="cuda").mul(2).repeat(B).contiguous()
    cache = KVCache4(B, n_keep + 66, H, dh)
    w = torch.randn((3 * d, d), generator=g, device="cuda", dtype=torch.float32) * 0.02
    lin = PackedLinear.from_fp32(w)
    del w
    y = torch.empty((M, 3 * d), dtype=torch.float16, device="cuda")
    q1 = rnd(B, d)
    o1 = torch.empty((B, d), dtype=torch.float16, device="cuda")

    def append():
        cache.reset()
        qb.quota_kv_quant_append(khat, vhat, B, N, H, dh, keep, n_keep, cache.desc)

    def decode_attn():
        cache.desc.len = n_keep + 65           # pruned prefix + 65 decoded tokens
        qb.quota_attention_decode(q1, cache.desc, o1)

    Md = float(M) * d
    cases = [
        ("quantize_act", lambda: qb.quota_quantize_act(x, M, d, d, qa, sa, sq, rq), 2.5 * Md, 0),
        ("rmsnorm_quantize_act", lambda: qb.quota_rmsnorm_quantize_act(x, M, d, d, gamma, 1e-5, qa, sa, sq, rq), 2.5 * Md, 0),
        ("silu_mul_quantize_act", lambda: qb.quota_silu_mul_quantize_act(gu, M, F, qa, sa), 4.5 * M * F, 0),
        ("rope_kv_quant", lambda: qb.quota_rope_kv_quant(qkv, M, H, dh, pos, cosT, sinT, N, q_rot, khat, vhat, kc, ks, vc, vs),
         Md * (6 + 6 + 1 + 1.0 / 16), 0),
        ("kv_quant_append", append, B * n_keep * d * (4 + 1 + 1.0 / 16), 0),
        ("attention_decode", decode_attn, B * (n_keep + 65) * (d + d / 16.0), 0),
        ("w4a4_gemm qkv", lambda: qb.quota_w4a4_gemm(qa, sa, M, lin.desc, y, 3 * d), 0, 2.0 * M * 3 * d * d),
    ]
    out = {}
    for name, fn, nbytes, ops in cases:
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        rec = dict(avg_us=round(us, 2))
        if nbytes:
            rec.update(GBps=round(nbytes / us / 1e3, 1), frac_hbm_peak=round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4))
        if ops:
            rec.update(TOPs=round(ops / us / 1e6, 1), frac_int8_peak=round(ops / us / 1e6 / PEAK_INT8_TOPS, 4))
        out[name] = rec
    return dict(shape=f"batch {B} x {N} tokens, d={d}, F={F} ({M} rows)", reps=reps, kernels=out)


def serving_decode(shape, stack, budgets, seed, steps=16):
    """Batched-serving shape end to end on the same weights: batch 16 x (576 + 128) tokens pruned
    prefill, then `steps` decode steps (random next-token embeddings) over the pruned 4-bit caches.
    Supplementary: decode tokens/s and the weight-streaming bound of a step."""
    import torch
    from paper_2604_17320_amd import workloads as wl
    from paper_2604_17320_amd.model import PrefillStack
    B, Nv, Nt = 16, shape.Nv, 128
    N = Nv + Nt
    big = PrefillStack(stack.layers, B, N, 0, Nv, budgets, decode_capacity=steps + 3)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed + 99)
    x0 = torch.randn((B * N, shape.d), generator=g, device="cuda", dtype=torch.float32).to(torch.float16)
    pos0 = torch.arange(N, dtype=torch.int32, device="cuda").repeat(B)
    big.run(x0, pos0)                           # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    big.run(x0, pos0)
    torch.cuda.synchronize()
    prefill_ms = (time.perf_counter() - t0) * 1e3
    xs = torch.randn((steps + 1, B, shape.d), generator=g, device="cuda", dtype=torch.float32).to(torch.float16)
    pn = torch.full((B,), N, dtype=torch.int32, device="cuda")
    big.decode(xs[0], pn)                       # warm-up step (also grows every cache by one row)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        pn = torch.full((B,), N + 1 + i, dtype=torch.int32, device="cuda")
        big.decode(xs[1 + i], pn)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    from paper_2604_17320_amd import binding as qb
    qb.quota_profile_begin(20 * len(stack.layers) + 16)
    big.decode(xs[0], torch.full((B,), N + 1 + steps, dtype=torch.int32, device="cuda"))
    kstats = qb.quota_profile_collect()
    gpu_ms = sum(v["total_ms"] for v in kstats.values())
    per_kernel = {k: round(v["total_ms"] * 1e3 / v["launches"], 2) for k, v in kstats.items()}
    wbytes = sum(l.weight_bytes() for l in stack.layers)
    kv_bytes = sum(B * c.len * (shape.d + shape.d // 16) for c in big.caches)
    return dict(shape=f"batch {B} x ({Nv} + {Nt}) tokens, {len(stack.layers)} layers", prefill_ms=round(prefill_ms, 2),
                prefill_tokens_per_s=round(B * N / prefill_ms * 1e3, 1), decode_steps=steps,
                decode_ms_per_step=round(ms, 3), decode_tokens_per_s=round(B / ms * 1e3, 1),
                decode_kernel_ms_per_step=round(gpu_ms, 3), decode_avg_us_per_kernel=per_kernel,
                weight_bytes_per_step=wbytes, kv_bytes_per_step=kv_bytes,
                hbm_bound_ms=round((wbytes + kv_bytes) / (PEAK_HBM_GBS * 1e9) * 1e3, 3),
                frac_hbm_peak=round((wbytes + kv_bytes) / (ms * 1e-3) / (PEAK_HBM_GBS * 1e9), 4))


def cpu_baseline(shape, stack, budgets, rope, sample_layers, seed):
    """The oracle, as it stands, on a bounded sample: a few layers of the stack, each fed a
    synthetic hidden state with the row count that layer sees in the real run."""
    import numpy as np
    import oracle
    from paper_2604_17320_amd import workloads as wl
    cos, sin = rope
    rows_in = []
    n, nv = shape.N, shape.Nv
    for K in budgets:
        rows_in.append((n, nv))
        k = nv if K < 0 else min(K, nv)
        n, nv = n - nv + k, k
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    t_sum, r_sum = 0.0, 0
    for l in sample_layers:
        L = stack.layers[l]
        W = oracle.LayerWeights(
            **{name: (getattr(L, name).codes.cpu().numpy(), getattr(L, name).plain_scales.cpu().numpy())
               for name in ("qkv", "o", "gu", "down")},
            gamma1=np.ones(shape.d, np.float32), gamma2=np.ones(shape.d, np.float32), eps=1e-5,
            H=shape.H, dh=shape.dh, F=shape.F)
        n, nv = rows_in[l]
        sh = wl.Shape("sample", shape.d, shape.H, shape.F, 1, shape.B, nv, n - nv, shape.n_outlier)
        x = wl.hidden_state(sh, seed + l)
        pos = wl.positions(sh)
        t0 = time.perf_counter()
        oracle.prefill_layer(W, x, pos, shape.B, n, 0, nv, budgets[l], cos, sin, prune_mid=True)
        t_sum += time.perf_counter() - t0
        r_sum += shape.B * n
    rows_total = sum(shape.B * n for n, _ in rows_in)
    est = t_sum * rows_total / r_sum                 # seconds for the whole stack, by row count
    return dict(value=shape.B * shape.N / est, unit="tokens/s", cores=threads, kind="oracle",
                sample=f"layers {list(sample_layers)} of {shape.layers} run in full ({t_sum:.2f} s, {r_sum} "
                       f"token-rows), scaled by token-rows to all layers ({rows_total} rows)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="c3", choices=["c1", "c2", "c3"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--profile-steps", type=int, default=3)
    ap.add_argument("--serving-shape", action="store_true",
                    help="also report (outside the timed region) per-kernel rates at the batch-16 serving "
                         "shape and the batch-16 prefill + decode steps on the same weights")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain elementwise copy of this many MiB (read + write), untimed: "
                         "the known-size kernel that HBM traffic counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (no sharding, no collectives); --gpus N>1 is not "
              "supported. Sequences are independent, so data parallelism over the batch would need no "
              "exchange step.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_17320_amd import binding as qb, workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    qb.lib()                                         # fails loudly if libquota.so is missing

    shape = {"c1": wl.CONFIGS[0], "c2": wl.CONFIGS[1], "c3": wl.CONFIGS[2]}[args.config]
    budgets = wl.schedule_for(shape)
    sample_layers = sorted({0, min(2, shape.layers - 1), shape.layers // 2, shape.layers - 1})
    stack, rope = build_stack(shape, args.seed, budgets, keep_plain_layers=() if args.no_cpu else sample_layers)
    x0 = torch.from_numpy(wl.hidden_state(shape, args.seed)).cuda()
    pos0 = torch.from_numpy(wl.positions(shape)).cuda()

    def step():
        return stack.run(x0, pos0)

    if args.calibration_copy_mib:
        src = torch.ones(args.calibration_copy_mib << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()

    graph = None
    if not args.no_graph:
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            graph.replay()
            torch.cuda.synchronize()
        except Exception as e:                       # noqa: BLE001 -- report and time eagerly instead
            print(f"bench.py: HIP graph capture failed ({e}); timing eager launches", file=sys.stderr)
            graph = None
    run = graph.replay if graph is not None else step

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    tokens = shape.B * shape.N
    value = tokens * args.steps / elapsed

    # eager timing for reference (launch overhead visible)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(max(1, args.steps // 5)):
        step()
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) * 1e3 / max(1, args.steps // 5)

    # per-kernel HIP-event timing over full eager steps.  An event pair around a launch reads the
    # kernel's run time plus the cost of the pair itself (2-4 us on this machine, measured below
    # with empty kernels).  The rates reported here use the RAW event time, so they are lower
    # bounds; `avg_us_net` has the measured pair cost taken off and brackets the kernel-trace
    # figure from the other side.
    bracket_ms, empty_kernel_ms = qb.quota_profile_bracket_ms(64)
    kernels_per_step = 20 * shape.layers
    qb.quota_profile_begin(kernels_per_step * args.profile_steps + 16)
    for _ in range(args.profile_steps):
        step()
    stats = qb.quota_profile_collect()
    kern = {}
    for name, s in stats.items():
        us = s["total_ms"] * 1e3 / s["launches"]
        kern[name] = dict(launches_per_step=s["launches"] // args.profile_steps, avg_us=round(us, 2),
                          avg_us_net=round(max(us - bracket_ms * 1e3, 0.0), 2),
                          step_ms=round(s["total_ms"] / args.profile_steps, 4),
                          GBps=round(s["bytes"] / (s["total_ms"] * 1e-3) / 1e9, 1) if s["total_ms"] else None,
                          TOPs=round(s["ops"] / (s["total_ms"] * 1e-3) / 1e12, 1) if s["ops"] else None)
    dom = max(stats, key=lambda k: stats[k]["total_ms"])
    ds = stats[dom]
    per_launch = dict(avg_launch_us=round(ds["total_ms"] * 1e3 / ds["launches"], 2),
                      avg_launch_us_net=round(max(ds["total_ms"] * 1e3 / ds["launches"] - bracket_ms * 1e3, 0.0), 2),
                      event_bracket_us=round(bracket_ms * 1e3, 2), empty_kernel_us=round(empty_kernel_ms * 1e3, 2),
                      launches_per_step=ds["launches"] // args.profile_steps)
    traffic_detail = measured_traffic(dom)
    traffic = traffic_detail["bytes_per_launch"] if traffic_detail else None     # HBM bytes per launch
    per_launch["traffic_detail"] = traffic_detail
    if ds["ops"] and dom.startswith("w4a4_gemm"):
        achieved = ds["ops"] / (ds["total_ms"] * 1e-3) / 1e12
        roofline = dict(kernel=dom, bound="mfma", achieved=round(achieved, 1), peak=PEAK_INT8_TOPS,
                        unit="TOP/s", frac=round(achieved / PEAK_INT8_TOPS, 4), traffic=traffic, **per_launch)
    else:
        achieved = ds["bytes"] / (ds["total_ms"] * 1e-3) / 1e9
        roofline = dict(kernel=dom, bound="hbm", achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(achieved / PEAK_HBM_GBS, 4), traffic=traffic, **per_launch)
    gemm_ops = sum(s["ops"] for n, s in stats.items() if n.startswith("w4a4_gemm"))
    gemm_ms = sum(s["total_ms"] for n, s in stats.items() if n.startswith("w4a4_gemm"))

    out = dict(metric="prefill_tokens_per_s", value=round(value, 1), unit="tokens/s", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=round(ms_per_step, 4),
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="int8",
               data="synthetic",
               config=dict(workload=f"{shape.name}: {shape.layers}-layer 7B-shaped W4A4 pruned prefill "
                                    f"(d={shape.d}, H={shape.H}, F={shape.F}), batch {shape.B}, "
                                    f"{shape.Nv} visual + {shape.Nt} text tokens, per-layer budgets "
                                    f"{budgets[0]}..{budgets[-1]} (mean keep "
                                    f"{sum(budgets) / len(budgets) / max(shape.Nv, 1):.3f}), 4-bit KV",
                           batch=shape.B, tokens_per_step=tokens, layers=shape.layers, seed=args.seed,
                           hip_graph=graph is not None),
               eager_ms_per_step=round(eager_ms, 4),
               roofline=roofline,
               gemm_all=dict(TOPs=round(gemm_ops / (gemm_ms * 1e-3) / 1e12, 1) if gemm_ms else None,
                             frac_int8_peak=round(gemm_ops / (gemm_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 4)
                             if gemm_ms else None, step_ms=round(gemm_ms / args.profile_steps, 4)),
               kernels=kern)
    if args.serving_shape:
        out["serving_shape_kernels"] = serving_shape_kernels(shape, args.seed)
        if args.config == "c3":
            out["serving_decode"] = serving_decode(shape, stack, budgets, args.seed)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(shape, stack, budgets, rope, sample_layers, args.seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
