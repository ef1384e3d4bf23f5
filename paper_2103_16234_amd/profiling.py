"""Turns rocprofv3 output of bench.py runs into the short text summaries kept under profiles/ and into the table of
measured HBM-side traffic that bench.py reports as `roofline.traffic`.

    python -m paper_2103_16234_amd.profiling traffic  DIR   # FETCH_SIZE / WRITE_SIZE passes -> profiles/conv_kernels_hbm_traffic.txt
                                                            #                                  + measured_traffic.json
    python -m paper_2103_16234_amd.profiling counters DIR   # SQ passes -> profiles/conv_kernels_sq_counters.txt
    python -m paper_2103_16234_amd.profiling stats    DIR   # kernel trace -> profiles/bench_five_layers_kernel_stats.txt

DIR holds, per layer tag T (cfg1 .. cfg5 for the benchmark layers, any other name for a --shape run):
    T_fetch/, T_write/, T_sq/   output directories of `rocprofv3 --pmc ... --output-format csv -d DIR/T_pass -o pmc -- python3 bench.py ...`
    T_fetch.json, ...           what the same bench.py run printed (its plan names the mapping the counters belong to)
    T.json                      (optional) the same bench.py command without the profiler: the undisturbed kernel time
and for `stats`: trace/ (rocprofv3 --kernel-trace --stats ... -o bench) and bench.json (the untraced default run).
Nothing here touches a GPU or the convolution's arithmetic.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
PROFILES = os.path.join(ROOT, "profiles")
TABLE = os.path.join(HERE, "measured_traffic.json")

PASSES = {
    "fetch": "FETCH_SIZE",
    "write": "WRITE_SIZE",
    "sq": "SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT SQ_VALU_MFMA_BUSY_CYCLES "
          "SQ_INSTS_MFMA GRBM_GUI_ACTIVE",
}
COPY_KIB = 65536.0       # bench.py's start-up copy: 64 MiB read, 64 MiB written


def bench_args(tag: str, shape: str | None) -> str:
    layer = f"--config {tag[3:]}" if shape is None else f"--shape {shape}"
    return f"python3 bench.py {layer} --no-layers --no-cpu --no-probes --steps 10 --warmup 2"


def command(tag: str, shape: str | None, which: str, root: str = "gpurun_out/prof") -> str:
    return (f"rocprofv3 --pmc {PASSES[which]} --output-format csv -d {root}/{tag}_{which} -o pmc -- "
            f"{bench_args(tag, shape)} > {root}/{tag}_{which}.json")


def _rows(directory: str):
    paths = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not paths:
        raise FileNotFoundError(f"no counter_collection.csv under {directory}")
    rows = []
    for p in paths:
        rows += list(csv.DictReader(open(p)))
    return rows


def _mean_by_counter(rows, name_part: str):
    agg = collections.defaultdict(list)
    for r in rows:
        if name_part in r["Kernel_Name"]:
            agg[r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in agg.items()}, {k: len(v) for k, v in agg.items()}


def _copy_reading(rows, counter: str):
    copies = [r for r in rows if "copyBuffer" in r["Kernel_Name"] and r["Counter_Name"] == counter]
    if not copies:
        return None
    largest = max(int(r["Grid_Size"]) for r in copies)     # the 64 MiB calibration copy is the largest copy of a run
    v = [float(r["Counter_Value"]) for r in copies if int(r["Grid_Size"]) == largest]
    return sum(v) / len(v)


def _bench_json(path: str):
    for line in reversed(open(path).read().splitlines()):
        line = line.strip()
        if line.startswith("{"):
            return json.loads(line)
    raise ValueError(f"no JSON line in {path}")


def _tags(directory: str, which: str):
    return sorted(os.path.basename(p)[: -len(f"_{which}.json")] for p in glob.glob(os.path.join(directory, f"*_{which}.json")))


def _layer_line(b):
    d = b["roofline"]
    return b["config"]["workload"].split(":")[0], d["algorithmic_bytes"], d["algorithmic_flops"], b["config"]["plan"]


def _shape_arg(b):
    # "name: N=.. C=.. H=.. W=.. K=.. R=.. S=.. pad=a,b stride 1, ..."
    f = dict(t.split("=") for t in b["config"]["workload"].split(": ", 1)[1].split(" stride")[0].split())
    return ",".join([f["N"], f["C"], f["H"], f["W"], f["K"], f["R"], f["S"]] + f["pad"].split(","))


def traffic(directory: str):
    tags = _tags(directory, "fetch")
    lines = ["HBM-side traffic of the convolution kernel per launch (rocprofv3 --pmc, KiB per dispatch, averaged over the",
             "dispatches of a run)", "", "commands, two runs per layer (from the repository root, on the MI355X box):"]
    table = {"note": "bytes per launch the L2s exchanged with the fabric, written by paper_2103_16234_amd/profiling.py from "
                     "rocprofv3 FETCH_SIZE / WRITE_SIZE runs of bench.py; plan = [kernel, variant, tile_pix, loader] measured",
             "layers": {}}
    body = []
    scale_f = scale_w = None
    for tag in tags:
        bf = _bench_json(os.path.join(directory, f"{tag}_fetch.json"))
        bw = _bench_json(os.path.join(directory, f"{tag}_write.json"))
        name, alg_bytes, _, plan = _layer_line(bf)
        assert plan == bw["config"]["plan"], f"{tag}: the two passes ran different mappings"
        shape = None if tag.startswith("cfg") and tag[3:].isdigit() else _shape_arg(bf)
        lines += ["  " + command(tag, shape, "fetch"), "  " + command(tag, shape, "write")]
        rf, rw = _rows(os.path.join(directory, f"{tag}_fetch")), _rows(os.path.join(directory, f"{tag}_write"))
        cf, cw = _copy_reading(rf, "FETCH_SIZE"), _copy_reading(rw, "WRITE_SIZE")
        if cf and cw:
            scale_f, scale_w = COPY_KIB / cf, COPY_KIB / cw
        if scale_f is None:
            raise ValueError(f"{tag}: no calibration copy found in the counter files")
        fe, nf = _mean_by_counter(rf, "conv_")
        wr, nw = _mean_by_counter(rw, "conv_")
        fb, wb = fe["FETCH_SIZE"] * 1024 * scale_f, wr["WRITE_SIZE"] * 1024 * scale_w
        dims = [int(v) for v in _shape_arg(bf).split(",")]
        n, c, h, w, k, r, s_, ph, pw = dims
        p, q = h + 2 * ph - r + 1, w + 2 * pw - s_ + 1
        alg_r, alg_w = 4 * (n * c * h * w + k * c * r * s_), 4 * n * k * p * q
        assert alg_r + alg_w == alg_bytes
        us = None
        if os.path.exists(os.path.join(directory, f"{tag}.json")):
            us = _bench_json(os.path.join(directory, f"{tag}.json"))["roofline"]["kernel_us"]
        body.append((tag, name, fe["FETCH_SIZE"], fb, alg_r, wr["WRITE_SIZE"], wb, alg_w, us, scale_f, scale_w, plan))
        table["layers"][",".join(str(d) for d in dims)] = {
            "layer": name, "fetch_bytes": int(fb), "write_bytes": int(wb), "algorithmic_bytes": alg_bytes,
            "plan": [plan["kernel"], plan["variant"], plan["tile_pix"], plan["loader"]]}
    lines += ["", "calibration: the plain 64 MiB device-to-device copy bench.py makes at start-up (the runtime's copyBuffer kernel: 65536 KiB",
              "read + 65536 KiB written), found in the same counter files: scale = 65536 / reading (FETCH_SIZE reads about half the copied",
              "bytes on this GPU, hence ~2; WRITE_SIZE ~1). Scaled bytes = reading x 1024 x scale.", ""]
    lines.append(f"{'layer':<34} {'FETCH KiB':>10} {'x':>6} {'read MB':>9} {'alg. MB':>9} {'ratio':>6} | {'WRITE KiB':>10} {'x':>6} "
                 f"{'write MB':>9} {'alg. MB':>9} {'ratio':>6} | {'total/alg.':>10} {'kernel us':>10} {'traffic GB/s':>12}")
    for tag, name, fk, fb, ar, wk, wb, aw, us, sf, sw, plan in body:
        rate = f"{(fb + wb) / us / 1e3:>12.0f}" if us else f"{'-':>12}"
        ust = f"{us:>10.2f}" if us else f"{'-':>10}"
        lines.append(f"{name[:34]:<34} {fk:>10.1f} {sf:>6.3f} {fb / 1e6:>9.2f} {ar / 1e6:>9.2f} {fb / ar:>6.2f} | {wk:>10.1f} {sw:>6.3f} "
                     f"{wb / 1e6:>9.2f} {aw / 1e6:>9.2f} {wb / aw:>6.2f} | {(fb + wb) / (ar + aw):>10.2f} {ust} {rate}")
    lines += ["", "mappings measured (kernel family, tile shape, pixel tile, loader):"]
    for tag, name, *_rest, plan in body:
        lines.append(f"  {name[:34]:<34} kernel {plan['kernel']} variant {plan['variant']} tile_pix {plan['tile_pix']} loader {plan['loader']} "
                     f"grid {plan['grid']} block {plan['block']}")
    lines += ["", "kernel us / traffic GB/s: the kernel's duration in an unprofiled run of the same command (HIP events, rotating buffers)",
              "and the counted bytes over it; '-' where no such run was kept.",
              "FETCH_SIZE counts what the L2s request from the fabric (Infinity Cache or HBM); a ratio above 1 is data fetched by more than",
              "one of the eight L2s or fetched again after eviction."]
    os.makedirs(PROFILES, exist_ok=True)
    open(os.path.join(PROFILES, "conv_kernels_hbm_traffic.txt"), "w").write("\n".join(lines) + "\n")
    json.dump(table, open(TABLE, "w"), indent=1)
    print("\n".join(lines))


def counters(directory: str):
    tags = _tags(directory, "sq")
    lines = ["Shader counters of the convolution kernel per launch (rocprofv3 --pmc, one pass, averages over the dispatches of a run)", "",
             "commands (from the repository root, on the MI355X box):"]
    body = []
    for tag in tags:
        b = _bench_json(os.path.join(directory, f"{tag}_sq.json"))
        name, _, flops, plan = _layer_line(b)
        shape = None if tag.startswith("cfg") and tag[3:].isdigit() else _shape_arg(b)
        lines.append("  " + command(tag, shape, "sq"))
        c, _ = _mean_by_counter(_rows(os.path.join(directory, f"{tag}_sq")), "conv_")
        us = None
        if os.path.exists(os.path.join(directory, f"{tag}.json")):
            us = _bench_json(os.path.join(directory, f"{tag}.json"))["roofline"]["kernel_us"]
        body.append((name, c, flops, plan, us))
    lines += ["", "Counters are sums over the chip (SQ_*: all 256 CUs; GRBM_GUI_ACTIVE: the 8 XCDs, so kernel cycles = GRBM_GUI_ACTIVE / 8).",
              "A v_mfma_f32_16x16x4_f32 occupies its SIMD's matrix unit for 32 cycles: MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (kernel cycles x 1024",
              "SIMDs). Counter collection slows short kernels down, so 'busy @ bench' divides the same busy cycles by the kernel's duration in an",
              "unprofiled run (HIP events, 2.4 GHz). per wave = instructions of that kind one wave issues.", ""]
    lines.append(f"{'layer':<28} {'waves':>7} {'kern cyc':>9} {'MFMA inst':>10} {'MFMA busy':>9} {'busy@bench':>10} {'useful':>7} "
                 f"{'VALU/wave':>9} {'LDS/wave':>9} {'MFMA/wave':>9} {'bank confl / LDS busy':>21} {'bench us':>9}")
    for name, c, flops, plan, us in body:
        cyc = c["GRBM_GUI_ACTIVE"] / 8
        waves = max(c["SQ_WAVES"], 1.0)
        busy = c["SQ_VALU_MFMA_BUSY_CYCLES"] / (cyc * 1024)
        at_bench = c["SQ_VALU_MFMA_BUSY_CYCLES"] / (us * 1e-6 * 2.4e9 * 1024) if us else float("nan")
        useful = flops / (c["SQ_INSTS_MFMA"] * 2048) if c.get("SQ_INSTS_MFMA") else float("nan")
        lines.append(f"{name[:28]:<28} {waves:>7.0f} {cyc:>9.0f} {c['SQ_INSTS_MFMA']:>10.0f} {busy:>9.3f} {at_bench:>10.3f} {useful:>7.3f} "
                     f"{c['SQ_INSTS_VALU'] / waves:>9.0f} {c['SQ_INSTS_LDS'] / waves:>9.0f} {c['SQ_INSTS_MFMA'] / waves:>9.0f} "
                     f"{c['SQ_LDS_BANK_CONFLICT']:>21.0f} {us if us else float('nan'):>9.2f}")
    lines += ["", "mappings measured:"]
    for name, c, flops, plan, us in body:
        lines.append(f"  {name[:28]:<28} kernel {plan['kernel']} variant {plan['variant']} tile_pix {plan['tile_pix']} loader {plan['loader']} "
                     f"grid {plan['grid']} block {plan['block']} lds {plan['lds_bytes']}")
    lines += ["", "useful = the layer's 2*N*K*P*Q*C*R*S over 2048 flops per issued MFMA (16-pixel tiles that hang over the end of a pixel tile and",
              "channel groups past C are the rest). SQ_BUSY_CYCLES and SQ_WAVE_CYCLES (per layer, in the order above):"]
    for name, c, *_ in body:
        lines.append(f"  {name[:28]:<28} SQ_BUSY_CYCLES {c['SQ_BUSY_CYCLES']:.0f}  SQ_WAVE_CYCLES {c['SQ_WAVE_CYCLES']:.0f}")
    os.makedirs(PROFILES, exist_ok=True)
    open(os.path.join(PROFILES, "conv_kernels_sq_counters.txt"), "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


def stats(directory: str):
    paths = glob.glob(os.path.join(directory, "trace", "**", "*kernel_stats.csv"), recursive=True)
    if not paths:
        raise FileNotFoundError(f"no kernel_stats.csv under {directory}/trace")
    rows = list(csv.DictReader(open(paths[0])))
    b = _bench_json(os.path.join(directory, "bench.json"))
    lines = ["rocprofv3 kernel-trace summary of the default benchmark run (headline layer, all five layers with both mappings, batch-scaled 1x1)",
             "command (on the MI355X box, from the repository root):",
             "  rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof/trace -o bench -- python3 bench.py",
             "source: bench_kernel_stats.csv, the library's kernels only (durations in ns)", "",
             f"{'kernel':<78} {'calls':>6} {'avg_ns':>10} {'min_ns':>9} {'max_ns':>9} {'stddev':>8}"]
    for r in rows:
        if "convfwd" in r["Name"]:
            name = r["Name"].replace("void convfwd::", "").replace("(convfwd::KernelArgs)", "")
            lines.append(f"{name[:78]:<78} {r['Calls']:>6} {float(r['AverageNs']):>10.0f} {r['MinNs']:>9} {r['MaxNs']:>9} {float(r['StdDev']):>8.0f}")
    lines += ["", "template arguments of conv_tap_mfma: <R, S, MT, NT, WK, WP, WC, GPC, OCC, XS, WS, VX, VW, direct loader>", "",
              "headline of the untraced run of the same command (bench.py's own HIP events):",
              f"  {b['config']['workload']}",
              f"  kernel {b['roofline']['kernel']}: {b['roofline']['kernel_us']:.2f} us per launch over {b['steps']} launches -> "
              f"{b['roofline']['achieved']:.2f} {b['roofline']['unit']} = {b['roofline']['frac']:.3f} of {b['roofline']['peak']} "
              f"({b['roofline']['bound']} roofline)", "",
              "layers of the same untraced run (default mapping | the cost model's own pick):"]
    for l in b.get("layers", []):
        m = l["cost_model_pick"]
        lines.append(f"  {l['layer']:<18} {l['kernel_us'] * 1000:>9.0f} ns ({l['gflops'] / 1e3:>7.2f} TFLOP/s, {l['gbs']:>6.0f} GB/s, "
                     f"{l['roofline']['frac']:.3f} of the {l['roofline']['bound']} roofline) variant {l['plan']['variant']} tile_pix "
                     f"{l['plan']['tile_pix']} loader {l['plan']['loader']} grid {l['plan']['grid']} | model: variant {m['plan']['variant']} tile_pix "
                     f"{m['plan']['tile_pix']} loader {m['plan']['loader']} {m['kernel_us'] * 1000:.0f} ns ({m['over_default']:.3f}x)")
    for r in b.get("batch_scaled_1x1", []):
        lines.append(f"  {r['layer']:<36} {r['kernel_us'] * 1000:>9.0f} ns ({r['tflops']:.2f} TFLOP/s, {r['gbs']:.0f} GB/s, "
                     f"{100 * r['frac_hbm_peak']:.1f} % of HBM peak)")
    os.makedirs(PROFILES, exist_ok=True)
    open(os.path.join(PROFILES, "bench_five_layers_kernel_stats.txt"), "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("traffic", "counters", "stats", "commands"):
        sys.exit(__doc__)
    if sys.argv[1] == "commands":     # the counter runs of one layer tag[=shape], one per line
        tag, _, shape = sys.argv[2].partition("=")
        for which in PASSES:
            print(command(tag, shape or None, which))
    else:
        {"traffic": traffic, "counters": counters, "stats": stats}[sys.argv[1]](sys.argv[2])
