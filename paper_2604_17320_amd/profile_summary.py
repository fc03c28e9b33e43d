#!/usr/bin/env python3
"""Condenses rocprofv3 CSV output of bench.py into the short text/JSON summaries kept under
profiles/.

    python -m paper_2604_17320_amd.profile_summary stats  <kernel_stats.csv>  [bench.json]
    python -m paper_2604_17320_amd.profile_summary traffic <fetch_counter_collection.csv> \
           <write_counter_collection.csv> <copy MiB> [bench.json]

`stats` prints the per-kernel table of a `--kernel-trace --stats` run next to bench.py's own
event-timed averages.  `traffic` turns two `--pmc` passes (FETCH_SIZE, then WRITE_SIZE, KiB per
dispatch) into HBM bytes per launch for each library kernel; both counters are scaled by what
they read for the plain elementwise copy of known size that bench.py ran in the same process
(`--calibration-copy-mib`), and the JSON goes to stdout.

    python -m paper_2604_17320_amd.profile_summary mfma <sq_counter_collection.csv> [bench.json]

    python -m paper_2604_17320_amd.profile_summary bandwidth <kernel_stats.csv> \
           <fetch_counter_collection.csv> <write_counter_collection.csv> <copy MiB> <bandwidth.json>

`bandwidth` does the same for a `bench.py --bandwidth-only` run (the bandwidth-bound kernels at the
batched-serving row count): per kernel the trace's average duration, the HBM bytes the two counter
passes read per launch, the algorithmic bytes, and the rate against the HBM peak.

`mfma` condenses one `--pmc` pass of SQ counters (SQ_INSTS_MFMA SQ_INSTS_VALU
SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_ACTIVE_INST_VALU SQ_WAVE_CYCLES SQ_WAIT_INST_ANY
SQ_WAVES) into one line per GEMM kernel class: MFMA instructions issued per launch and what they
amount to against the int8 dense peak over the dispatch's own duration, vector instructions per
MFMA, and the busy / wait shares the counters give.
"""
import collections
import csv
import json
import re
import sys

# profiler kernel name (substring) -> kernel class name used by the library's own timing
CLASSES = [
    ("w4a4_gemm_kernelILi2ELi2E", "w4a4_gemm_64x256"),
    ("w4a4_gemm_kernelILi2ELi1ELi4ELi2ELb1ELb0E", "w4a4_gemm_64x128"),
    ("w4a4_gemm_kernelILi2ELi1ELi3ELi0ELb0ELb0E", "w4a4_gemm_64x128_lean"),
    ("w4a4_gemm_kernelILi1ELi1ELi4E", "w4a4_gemm_32x128"),
    ("w4a4_gemm_kernelILi1ELi1ELi8E", "w4a4_gemm_32x128_deep"),
    ("w4a4_gemm_kernel", "w4a4_gemm_other"),
    ("w4a4_gemv16_kernel", "w4a4_gemm_rows16"),
    ("silu_mul_quantize_act_kernel", "silu_mul_quantize_act"),
    ("rmsnorm_quantize_act_kernel", "rmsnorm_quantize_act"),
    ("quantize_act_kernel", "quantize_act"),
    ("rope_kv_quant_mha_kernel", "rope_kv_quant"),
    ("rope_kv_quant_kernel", "rope_kv_quant"),
    ("kv_quant_append_kernel", "kv_quant_append"),
    ("attn_fwd_kernel", "attention_fwd"),
    ("colmass_reduce_kernel", "attention_colmass_reduce"),
    ("colmass_kernel", "attention_colmass"),
    ("score_topk_kernel", "score_tokens"),
    ("topk_kernel", "topk_prune"),
    ("compact_rows_kernel", "compact_rows"),
    ("decode_attention_kernel", "attention_decode"),
    ("kv_append_rows_kernel", "kv_append_rows"),
    ("quantize_weights_kernel", "quantize_weights"),
    ("pack_weights_kernel", "pack_weights"),
]


def classify(name):
    for key, cls in CLASSES:
        if key in name:
            return cls
    return None


def load_bench(path):
    if not path:
        return None
    with open(path) as f:
        lines = [l for l in f.read().splitlines() if l.startswith("{")]
    return json.loads(lines[-1]) if lines else None


def stats(csv_path, bench_path=None):
    bench = load_bench(bench_path)
    agg = collections.OrderedDict()
    for r in csv.DictReader(open(csv_path)):
        cls = classify(r["Name"])
        if cls is None:
            continue
        a = agg.setdefault(cls, [0, 0.0])
        a[0] += int(r["Calls"])
        a[1] += float(r["TotalDurationNs"])
    total = sum(a[1] for a in agg.values())
    print(f"{'kernel':28s} {'calls':>7s} {'avg us (trace)':>15s} {'share':>7s} {'events: avg us':>15s} {'net of pair':>12s}")
    for cls, (calls, ns) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        k = (bench and bench["kernels"].get(cls)) or {}
        ev, net = k.get("avg_us"), k.get("avg_us_net")
        print(f"{cls:28s} {calls:7d} {ns / calls / 1e3:15.2f} {100 * ns / total:6.1f}% "
              f"{'' if ev is None else format(ev, '15.2f')} {'' if net is None else format(net, '12.2f')}")
    if bench:
        print(f"\nbench.py line (plain run of the same command, no profiler attached): {bench['value']} {bench['unit']}, {bench['ms_per_step']} ms/step, "
              f"roofline {json.dumps(bench['roofline'])}")


def per_kernel(csv_path, counter):
    """{class: [values per dispatch]} plus the copy kernel's values."""
    vals, copy = collections.defaultdict(list), []
    for r in csv.DictReader(open(csv_path)):
        if r["Counter_Name"] != counter:
            continue
        name, v = r["Kernel_Name"], float(r["Counter_Value"])
        cls = classify(name)
        if cls:
            vals[cls].append(v)
        elif "elementwise_kernel" in name and "AUnaryFunctor" in name:
            copy.append((int(r["Grid_Size"]), v))      # torch.mul(src, 1.0, out=dst), 4 floats per thread
    return vals, copy


def traffic(fetch_csv, write_csv, copy_mib, bench_path=None):
    bench = load_bench(bench_path)
    copy_bytes = int(copy_mib) << 20
    out = dict(counters="FETCH_SIZE, WRITE_SIZE (KiB per dispatch), one rocprofv3 --pmc pass each",
               calibration={}, kernels={})
    scale = {}
    for tag, path, ctr in (("fetch", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        vals, copy = per_kernel(path, ctr)
        big = [v for g, v in copy if g == copy_bytes // 16]          # the copy itself, by its grid size
        if len(big) != 1:
            raise SystemExit(f"expected one calibration copy in {path}, found {len(big)}")
        read_kib = big[0]
        scale[tag] = copy_bytes / (read_kib * 1024.0)
        out["calibration"][tag] = dict(copy_bytes=copy_bytes, counter_kib=read_kib, scale=round(scale[tag], 4))
        for cls, v in vals.items():
            rec = out["kernels"].setdefault(cls, {})
            rec[f"{tag}_bytes"] = round(sum(v) / len(v) * 1024.0 * scale[tag])
            rec[f"{tag}_dispatches"] = len(v)
    if bench:
        for cls, rec in out["kernels"].items():
            k = bench["kernels"].get(cls)
            if k and k.get("GBps") and k.get("avg_us"):      # GBps is algorithmic bytes / raw event time
                rec["algorithmic_bytes"] = round(k["GBps"] * 1e9 * k["avg_us"] * 1e-6)
    print(json.dumps(out, indent=1))


def bandwidth_case(name):
    """Kernel symbol -> the case name bench.py's bandwidth_kernels block uses."""
    cls = classify(name)
    if cls in ("quantize_act", "rmsnorm_quantize_act") and (cls + "_kernelILb1E") in name:
        return cls + " (+ m_mag, m_res)"
    return cls


def bandwidth(stats_csv, fetch_csv, write_csv, copy_mib, bench_path):
    bench = load_bench(bench_path)["bandwidth_kernels"]
    cases = bench["kernels"]
    copy_bytes = int(copy_mib) << 20
    dur = collections.defaultdict(lambda: [0, 0.0])
    for r in csv.DictReader(open(stats_csv)):
        c = bandwidth_case(r["Name"])
        if c in cases:
            dur[c][0] += int(r["Calls"])
            dur[c][1] += float(r["TotalDurationNs"])
    hbm = collections.defaultdict(dict)
    scales = {}
    for tag, path, ctr in (("fetch", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        vals, copy = collections.defaultdict(list), []
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != ctr:
                continue
            name, v = r["Kernel_Name"], float(r["Counter_Value"])
            c = bandwidth_case(name)
            if c in cases:
                vals[c].append(v)
            elif "elementwise_kernel" in name and "AUnaryFunctor" in name and int(r["Grid_Size"]) == copy_bytes // 16:
                copy.append(v)
        if not copy:
            raise SystemExit(f"no calibration copy in {path}")
        # (the block's own reference case is the same copy again: every match moved copy_bytes each way)
        scales[tag] = copy_bytes / (sum(copy) / len(copy) * 1024.0)
        for c, v in vals.items():
            v = sorted(v)[len(v) // 2:]               # the warm-up launch of a case may differ; upper half
            hbm[c][tag] = sum(v) / len(v) * 1024.0 * scales[tag]
    print(f"shape: {bench['shape']}")
    print(f"counter scale (known-size copy of {copy_mib} MiB): FETCH_SIZE x {scales['fetch']:.4f}, WRITE_SIZE x {scales['write']:.4f}")
    print(f"{'kernel':40s} {'calls':>5s} {'avg us (trace)':>14s} {'algorithmic MB':>14s} {'HBM fetch MB':>12s} {'HBM write MB':>12s} "
          f"{'GB/s':>8s} {'of 8 TB/s':>9s} {'events: us':>10s}")
    for c, k in cases.items():
        if c not in dur:
            continue
        calls, ns = dur[c]
        us = ns / calls / 1e3
        alg = k["MB"] * 1e6
        print(f"{c:40s} {calls:5d} {us:14.2f} {alg / 1e6:14.1f} {hbm[c].get('fetch', float('nan')) / 1e6:12.1f} "
              f"{hbm[c].get('write', float('nan')) / 1e6:12.1f} {alg / us / 1e3:8.0f} {alg / us / 1e3 / 8000.0:9.3f} {k['avg_us']:10.2f}")
    print("\nGB/s = algorithmic bytes (inputs once + outputs once, 4-bit data as half bytes) / the trace's average duration;\n"
          "events: us = what bench.py's own event pair around the same launches read in the plain run.")


def mfma(csv_path, bench_path=None):
    bench = load_bench(bench_path)
    per = collections.defaultdict(lambda: collections.defaultdict(list))     # class -> counter -> values
    dur = collections.defaultdict(dict)                                      # class -> dispatch id -> ns
    for r in csv.DictReader(open(csv_path)):
        cls = classify(r["Kernel_Name"])
        if cls is None or not cls.startswith("w4a4_gemm"):
            continue
        per[cls][r["Counter_Name"]].append(float(r["Counter_Value"]))
        dur[cls][r["Dispatch_Id"]] = float(r["End_Timestamp"]) - float(r["Start_Timestamp"])
    mean = lambda v: sum(v) / len(v) if v else float("nan")
    print("per launch, mean over the dispatches of each GEMM kernel class (durations are those of the counter run, "
          "which serialises kernels and is slower than a plain run)")
    print(f"{'kernel':24s} {'launches':>8s} {'us':>7s} {'MFMA inst':>10s} {'issued TOP/s':>12s} {'of int8 peak':>12s} "
          f"{'VALU/MFMA':>9s} {'MFMA busy':>9s} {'VALU active':>11s} {'waiting':>8s}")
    for cls, c in sorted(per.items()):
        n = len(dur[cls])
        us = mean(list(dur[cls].values())) / 1e3
        m, v = mean(c["SQ_INSTS_MFMA"]), mean(c["SQ_INSTS_VALU"])
        tops = m * 65536.0 / (us * 1e-6) / 1e12            # one v_mfma_i32_32x32x32_i8 = 32*32*32 MACs
        busy_cu, wave_cyc = mean(c["SQ_BUSY_CU_CYCLES"]), mean(c["SQ_WAVE_CYCLES"])
        print(f"{cls:24s} {n:8d} {us:7.1f} {m:10.0f} {tops:12.1f} {tops / 5000.0:12.3f} {(v - m) / m:9.1f} "
              f"{mean(c['SQ_VALU_MFMA_BUSY_CYCLES']) / (4.0 * busy_cu):9.3f} {mean(c['SQ_ACTIVE_INST_VALU']) / wave_cyc:11.3f} "
              f"{mean(c['SQ_WAIT_INST_ANY']) / wave_cyc:8.3f}")
    print("\nMFMA inst: v_mfma_i32_32x32x32_i8 issued (all waves); issued TOP/s = MFMA inst * 65536 ops / duration (includes the\n"
          "rows and columns a tile pads); VALU/MFMA: other vector instructions per MFMA (SQ_INSTS_VALU counts the MFMAs too);\n"
          "MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs * SQ_BUSY_CU_CYCLES); VALU active, waiting = SQ_ACTIVE_INST_VALU, SQ_WAIT_INST_ANY\n"
          "over SQ_WAVE_CYCLES (share of wave lifetime).")
    if bench:
        g = bench.get("gemm_all", {})
        print(f"\nplain run of bench.py: GEMMs {g.get('TOPs')} TOP/s algorithmic = {g.get('frac_int8_peak')} of the int8 peak, "
              f"{g.get('step_ms')} ms of a {bench['ms_per_step']} ms step")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(*sys.argv[2:4])
    elif len(sys.argv) >= 3 and sys.argv[1] == "mfma":
        mfma(*sys.argv[2:4])
    elif len(sys.argv) >= 7 and sys.argv[1] == "bandwidth":
        bandwidth(*sys.argv[2:7])
    elif len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        traffic(*sys.argv[2:6])
    else:
        raise SystemExit(__doc__)
