"""Turns rocprofv3 output of bench.py runs into the short text summaries kept under profiles/ and into the table of
measured HBM-side traffic that bench.py reports as `roofline.traffic`.

    python -m paper_2103_16234_amd.profiling traffic  DIR   # FETCH_SIZE / WRITE_SIZE passes -> profiles/conv_kernels_hbm_traffic.txt
                                                            #                                  + measured_traffic.json
    python -m paper_2103_16234_amd.profiling counters DIR   # SQ passes -> profiles/conv_kernels_sq_counters.txt
    python -m paper_2103_16234_amd.profiling stats    DIR   # kernel trace -> profiles/bench_five_layers_kernel_stats.txt
    python -m paper_2103_16234_amd.profiling split_c | paper_shapes | short_reductions  FILE   # what bench.py printed with the
                                                            # option of that name -> the summary of that measurement
    python -m paper_2103_16234_amd.profiling sweep FILE...  # bench.py --sweep outputs (one, or one per filter size)
    python -m paper_2103_16234_amd.profiling holdout FILE...   # one bench.py --holdout SEED output per seed

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
    name = b["config"]["workload"].split(":")[0]
    if name.startswith("shape_"):      # a --shape run: say what the layer is
        n, c, h, w, k, r, s_, _, _ = (int(v) for v in _shape_arg(b).split(","))
        name = f"{r}x{s_} N{n} C{c} {h}x{w} K{k}"
    return name, d["algorithmic_bytes"], d["algorithmic_flops"], b["config"]["plan"]


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
            "plan": [plan["kernel"], plan["variant"], plan["tile_pix"], plan["loader"], plan.get("order", 0)]}
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
        useful = flops / (c["SQ_VALU_MFMA_BUSY_CYCLES"] * 64) if c.get("SQ_VALU_MFMA_BUSY_CYCLES") else float("nan")
        lines.append(f"{name[:28]:<28} {waves:>7.0f} {cyc:>9.0f} {c['SQ_INSTS_MFMA']:>10.0f} {busy:>9.3f} {at_bench:>10.3f} {useful:>7.3f} "
                     f"{c['SQ_INSTS_VALU'] / waves:>9.0f} {c['SQ_INSTS_LDS'] / waves:>9.0f} {c['SQ_INSTS_MFMA'] / waves:>9.0f} "
                     f"{c['SQ_LDS_BANK_CONFLICT']:>21.0f} {us if us else float('nan'):>9.2f}")
    lines += ["", "mappings measured:"]
    for name, c, flops, plan, us in body:
        lines.append(f"  {name[:28]:<28} kernel {plan['kernel']} variant {plan['variant']} tile_pix {plan['tile_pix']} loader {plan['loader']} "
                     f"grid {plan['grid']} block {plan['block']} lds {plan['lds_bytes']}")
    lines += ["", "useful = the layer's 2*N*K*P*Q*C*R*S over 64 flops per busy cycle of a matrix unit (2048 per v_mfma_f32_16x16x4_f32 = 32 cycles, 512 per",
              "v_mfma_f32_4x4x1_16B_f32 = 8 cycles; 16-pixel tiles that hang over the end of a pixel tile and channel groups past C are the rest). SQ_BUSY_CYCLES and SQ_WAVE_CYCLES (per layer, in the order above):"]
    for name, c, *_ in body:
        lines.append(f"  {name[:28]:<28} SQ_BUSY_CYCLES {c['SQ_BUSY_CYCLES']:.0f}  SQ_WAVE_CYCLES {c['SQ_WAVE_CYCLES']:.0f}")
    os.makedirs(PROFILES, exist_ok=True)
    open(os.path.join(PROFILES, "conv_kernels_sq_counters.txt"), "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))
    _mfma_utilisation(body, [command(t, None, "sq") for t in tags if t in ("cfg3", "cfg5")])


# The same two figures as measured with the kernels of commit 9ec1455 (registers-or-direct loaders only, per-lane integer division in the
# prologue): layer -> (mapping, MFMA busy under the profiler, MFMA busy at the benchmark duration, benchmark us, useful fraction).
EARLIER_MFMA = {
    "cfg3_3x3_c64_56": ("variant 7 tile_pix 112 loader 2", 0.375, 0.495, 23.75, 1.000),
    "cfg5_3x3_c512_14": ("variant 6 tile_pix 196 loader 1", 0.760, 0.781, 255.58, 0.942),
}


def _mfma_utilisation(body, commands):
    lines = ["Matrix-unit utilisation of the compute-bound benchmark layers (rocprofv3 --pmc, averages per dispatch of the convolution kernel)",
             "commands:"] + ["  " + c for c in commands]
    lines += ["", "MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 x 1024 SIMDs); a v_mfma_f32_16x16x4_f32 holds its SIMD's matrix unit for",
              "32 cycles. 'at bench' divides the same busy cycles by the kernel's duration in the unprofiled run (HIP events, 2.4 GHz); counter",
              "collection slows the short kernel down. useful = the layer's flops over 64 per busy cycle (the four-pixel tail tiles of the",
              "current kernels run v_mfma_f32_4x4x1_16B_f32: 8 cycles, 512 flops).", "",
              f"{'layer':<20} {'kernels':<10} {'mapping':<34} {'busy':>6} {'at bench':>9} {'useful':>7} {'bench us':>9}"]
    for name, c, flops, plan, us in body:
        if name not in EARLIER_MFMA:
            continue
        m, busy0, bench0, us0, useful0 = EARLIER_MFMA[name]
        useful = flops / (c["SQ_VALU_MFMA_BUSY_CYCLES"] * 64)
        lines.append(f"{name:<20} {'9ec1455':<10} {m:<34} {busy0:>6.3f} {bench0:>9.3f} {useful0:>7.3f} {us0:>9.2f}")
        cyc = c["GRBM_GUI_ACTIVE"] / 8
        now = f"variant {plan['variant']} tile_pix {plan['tile_pix']} loader {plan['loader']}"
        lines.append(f"{name:<20} {'this tree':<10} {now:<34} {c['SQ_VALU_MFMA_BUSY_CYCLES'] / (cyc * 1024):>6.3f} "
                     f"{c['SQ_VALU_MFMA_BUSY_CYCLES'] / (us * 1e-6 * 2.4e9 * 1024):>9.3f} {useful:>7.3f} {us:>9.2f}")
    lines += ["", "The achieved fraction of the fp32 MFMA peak is 'at bench' x useful (x the share of the 256 CUs that hold a work-group).",
              "Every counter of the same runs, for all five layers: conv_kernels_sq_counters.txt."]
    _write("conv_kernels_mfma_utilisation.txt", lines)


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
    lines += ["", "template arguments of conv_tap_mfma: <R, S, MT, NT, WK, WP, WC, GPC, OCC, XS, WS, VX, VW, direct loader, loader waves>", "",
              "headline of the untraced run of the same command (bench.py's own HIP events):",
              f"  {b['config']['workload']}",
              f"  kernel {b['roofline']['kernel']}: {b['roofline']['kernel_us']:.2f} us per launch over {b['steps']} launches -> "
              f"{b['roofline']['achieved']:.2f} {b['roofline']['unit']} = {b['roofline']['frac']:.3f} of {b['roofline']['peak']} "
              f"({b['roofline']['bound']} roofline)", "",
              "layers of the same untraced run (the planner's mapping; the library keeps no table of measured mappings):"]
    for l in b.get("layers", []):
        lines.append(f"  {l['layer']:<18} {l['kernel_us'] * 1000:>9.0f} ns ({l['gflops'] / 1e3:>7.2f} TFLOP/s, {l['gbs']:>6.0f} GB/s, "
                     f"{l['roofline']['frac']:.3f} of the {l['roofline']['bound']} roofline) variant {l['plan']['variant']} tile_pix "
                     f"{l['plan']['tile_pix']} loader {l['plan']['loader']} grid {l['plan']['grid']}")
    for r in b.get("batch_scaled_1x1", []):
        lines.append(f"  {r['layer']:<36} {r['kernel_us'] * 1000:>9.0f} ns ({r['tflops']:.2f} TFLOP/s, {r['gbs']:.0f} GB/s, "
                     f"{100 * r['frac_hbm_peak']:.1f} % of HBM peak)")
    os.makedirs(PROFILES, exist_ok=True)
    open(os.path.join(PROFILES, "bench_five_layers_kernel_stats.txt"), "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


FAMILY = {0: "generic", 1: "tap", 2: "pointwise", 3: "panel"}
LOADER = {1: " R", 2: " D", 3: " W", 4: " D4"}
PLAN_NOTE = ("plan: family, variant, tile_pix (panel: work-groups per channel tile), grid, block, loader of the tap family (R: through the\n"
             "registers, D: direct to LDS, W: direct by loader waves, D4: direct into a ring of four staging copies).")


def _plan(p):
    return f"{FAMILY[p[0]]} v{p[1]} {p[2]} g{p[3]} b{p[4]}" + (LOADER.get(p[5], "") if len(p) > 5 else "")


def _write(name, lines):
    os.makedirs(PROFILES, exist_ok=True)
    open(os.path.join(PROFILES, name), "w").write("\n".join(lines) + "\n")
    print("\n".join(lines[-8:]))


def _geomean(values):
    import math
    values = list(values)
    return math.exp(sum(math.log(v) for v in values) / len(values))


def sweep(paths):
    """bench.py --no-layers --no-cpu --sweep [SUBSTR] [--find] > path; several outputs (one per filter size) are joined"""
    import statistics
    rows = [r for p in paths for r in _bench_json(p)["sweep"]]
    found = all("found_us" in r for r in rows)
    lines = [f"Second workload: the synthetic shape sweep ({len(rows)} layers inside the ranges of the paper's evaluation, Section 4 / Table 1:",
             "batch 1, 8, 16, 32, 64, 128, 256; maps 7..224; 16..2048 filters; 1x1 / 3x3 / 5x5 with \"same\" padding; shapes from",
             "paper_2103_16234_amd.inputs.sweep_shapes, tensors of at most 2^25 elements), HIP-event time per launch over rotating buffer",
             "sets on one MI355X, each layer spot-checked against the oracle on 128 outputs."
             + (" Two mappings per layer: the planner's default," if found else ""),
             ("and the one conv_fwd_find measures to be fastest (cold-cache timing with a 512 MiB flush buffer); each of the two is timed"
              if found else "The planner's default mapping."),
             ("twice in turn (default, found, default, found) and its faster run counts: whichever runs right after the search's burst of\n"
              "launches finds the clocks up, worth up to 20 % on layers of a few microseconds." if found else ""),
             "Command (from the repository root):",
             "  python3 bench.py --no-layers --no-cpu --sweep" + (" --find" if found else "") + " > gpurun_out/prof/sweep.json"
             + ("      (run as three: --sweep sweep_1x1, sweep_3x3, sweep_5x5)" if len(paths) > 1 else ""),
             "bound/frac: the slower of the two roofline times (157.3 TFLOP/s fp32 MFMA, 8 TB/s HBM) over the measured time.", PLAN_NOTE, ""]
    head = f"{'layer':<36}{'us':>8} {'TFLOP/s':>8} {'GB/s':>7} bound   frac  {'default plan':<30}"
    lines.append(head + (" |  found us   frac  found plan" if found else ""))
    for r in rows:
        line = (f"{r['shape']:<36}{r['kernel_us']:8.1f} {r['tflops']:8.2f} {r['gbs']:7.0f} {r['bound']:<5} {r['frac']:6.3f}  "
                f"{_plan(r['plan']):<30}")
        if found:
            line += f" | {r['found_us']:9.1f} {r['found_frac']:6.3f}  {_plan(r['found_plan'])}"
        lines.append(line)
    lines.append("")
    ok = True
    for f in ("1x1", "3x3", "5x5"):
        rs = [r for r in rows if f"_{f}_" in r["shape"]]
        big = [r for r in rs if int(r["shape"].split("_n")[1].split("_")[0]) >= 32]
        text = (f"{f}: {len(rs)} layers; default plans: median fraction {statistics.median(r['frac'] for r in rs):.3f}, batch >= 32: "
                f"median {statistics.median(r['frac'] for r in big):.3f}, best {max(r['frac'] for r in big):.3f}")
        if found:
            gm = _geomean(r["kernel_us"] / min(r["found_us"], r["kernel_us"]) for r in rs)
            text += (f"; found plans: batch >= 32 median {statistics.median(max(r['found_frac'], r['frac']) for r in big):.3f}, best "
                     f"{max(r['found_frac'] for r in big):.3f}; default / found time, geometric mean {gm:.3f}")
        lines.append(text)
        ok &= all(r["parity_ok"] and r.get("found_parity_ok", True) for r in rs)
    lines.append(f"All {len(rows)} layers within tolerance on the sampled outputs." if ok else "PARITY FAILURES")
    _write("synthetic_shape_sweep.txt", lines)


def holdout(paths):
    """bench.py --no-cpu --no-layers --holdout SEED > path, one path per seed"""
    runs = [_bench_json(p)["holdout"] for p in paths]
    lines = ["Planner check on layers it was not fitted on: 40 random layers per seed inside the paper's ranges but off the synthetic",
             "sweep grid (batch 1, 2, 4, 16, 64; 16...640 channels; maps 7...112; 24...768 filters; 1x1 / 3x3 / 5x5), each timed on one",
             "MI355X with the default mapping (conv_fwd) and with the mapping conv_fwd_find measures to be fastest (cold-cache timing),",
             "HIP events over rotating buffer sets, the found mapping spot-checked against the oracle on 64 outputs. Each of the two",
             "mappings is timed twice in turn (default, found, default, found) and its faster run counts (a run right after the search's",
             "burst of launches finds the clocks up, worth up to 20 % on layers of a few microseconds).",
             "Commands (from the repository root), one per seed:",
             "  python3 bench.py --no-cpu --no-layers --holdout SEED > gpurun_out/prof/holdout_SEED.json      (SEED = "
             + ", ".join(str(h["seed"]) for h in runs) + ")",
             "frac: fraction of the binding roofline (157.3 TFLOP/s fp32 MFMA or 8 TB/s HBM) with the default mapping.", PLAN_NOTE, ""]
    for h in runs:
        ok = all(r["found_parity_ok"] for r in h["layers"])
        lines.append(f"seed {h['seed']}: default / found time, geometric mean {h['default_over_found_geomean']:.3f}, worst "
                     f"{h['default_over_found_worst']:.2f}; all found mappings within tolerance: {ok}")
        lines.append(f"  {'layer':<34} {'default us':>10} {'frac':>6}  {'default plan':<30} {'found us':>9}  found plan")
        for r in h["layers"]:
            lines.append(f"  {r['shape']:<34} {r['default_us']:>10.1f} {r['frac']:>6.3f}  {_plan(r['default_plan']):<30} {r['found_us']:>9.1f}  "
                         f"{_plan(r['found_plan'])}")
        lines.append("")
    _write("holdout_layers_default_vs_found.txt", lines)


def split_c(path: str):
    """bench.py --no-layers --no-cpu --split-c > path"""
    rows = _bench_json(path)["split_c"]
    lines = ["Channel splitting across work-groups (conv_fwd_split_c: the tap kernel writes one partial output per channel share into the",
             "caller's workspace, a second kernel adds the shares in order and applies the epilogue) against the single-kernel default",
             "(conv_fwd), on every layer of the synthetic shape grid and of the paper's profiled shapes (Tables 3-5) for which the splitting",
             "planner (conv_fwd_plan_split_c) asks for more than one share. One MI355X, HIP-event time per call over 400 calls on rotating",
             "buffer sets, both launches of the split mode included; each layer spot-checked against the oracle on 128 outputs.",
             "Command (from the repository root):", "  python3 bench.py --no-layers --no-cpu --split-c > gpurun_out/prof/split_c.json",
             "plan: family, variant, tile_pix, grid (work-groups, shares included), block, loader (R / D / W as in the sweep summary).", "",
             f"{'layer':<32} {'default us':>10}  {'default plan':<28} {'split us':>8}  {'split plan':<28} {'shares':>6} {'workspace':>10} {'speed-up':>8} parity"]
    for r in rows:
        lines.append(f"{r['shape']:<32} {r['default_us']:>10.1f}  {_plan(r['default_plan']):<28} {r['split_us']:>8.1f}  {_plan(r['split_plan']):<28} "
                     f"{r['c_splits']:>6} {r['workspace_bytes'] / 1e6:>8.1f}MB {r['default_us'] / r['split_us']:>7.2f}x "
                     f"{'ok' if r['split_parity_ok'] else 'FAIL'}")
    if rows:
        ups = [r["default_us"] / r["split_us"] for r in rows]
        lines += ["", f"{len(rows)} layers split; speed-up over the default: geometric mean {_geomean(ups):.2f}x, range {min(ups):.2f}x .. {max(ups):.2f}x."]
    _write("channel_splitting_layers.txt", lines)


def paper_shapes(path: str):
    """bench.py --no-layers --no-cpu --paper-shapes > path"""
    rows = _bench_json(path)["paper_shapes"]
    lines = ["Fused kernels vs. the opt-in two-stage scheme on the seven shapes of the paper's kernel-profile tables (Tables 3-5; batch 1",
             "except 5x5 B), HIP-event time per call over rotating buffer sets, one MI355X. Command (from the repository root):",
             "  python3 bench.py --no-layers --no-cpu --paper-shapes > gpurun_out/prof/paper_shapes.json",
             "The last two columns are the paper's own figures for its kernels and for the best vendor-library algorithm on a",
             "V100: context from another machine, not a target.", "",
             f"{'shape':<8} {'N,C,H,W,K,R,S,pad':<26} {'fused us':>9} {'plan':>14} {'two-stage us':>13} {'paper us':>9} {'vendor us':>10}  parity"]
    for r in rows:
        d = r["dims"]
        dims = ",".join(str(d[k]) for k in ("N", "C", "H", "W", "K", "R", "S", "pad_h"))
        p = r["fused_plan"]
        lines.append(f"{r['shape']:<8} {dims:<26} {r['fused_us']:>9.2f} {'k%d v%d g%d' % (p['kernel'], p['variant'], p['grid']):>14} "
                     f"{r['two_stage_us']:>13.2f} {r['paper_two_stage_us_v100']:>9.2f} {r['paper_best_vendor_us_v100']:>10.2f}  "
                     f"{r['fused_parity_ok'] and r['two_stage_parity_ok']}")
    lines += ["", "plan: k1 = tap kernel, k2 = pointwise kernel, k3 = panel kernel, v = variant index, g = work-groups"]
    _write("paper_profile_shapes_fused_vs_two_stage.txt", lines)


def short_reductions(path: str):
    """bench.py --no-layers --no-cpu --short-reductions > path"""
    rows = _bench_json(path)["short_reductions"]
    lines = ["fp32 MFMA against plain vector fp32 FMA on layers with a short reduction (C*R*S of 27 ... 400), one MI355X, HIP-event time per",
             "launch over 500 launches on rotating buffer sets; both checked against the oracle on 128 outputs.",
             "  mfma: the library's default mapping (tap family: LDS halo tile and filter block, v_mfma_f32_16x16x4_f32)",
             "  valu: the generic kernel (one output per thread, v_fma_f32, no LDS; the only plain-FMA kernel of the library - it has no",
             "        register blocking, so this is vector FMA as the definition gives it, not the best a vector-FMA kernel could do)",
             "Command (from the repository root):",
             "  python3 bench.py --no-layers --no-cpu --short-reductions > gpurun_out/prof/short.json", "",
             f"{'layer':<52} {'C*R*S':>6} {'mfma us':>8} {'valu us':>8} {'valu/mfma':>9}  default plan            parity"]
    for r in rows:
        p = r["default_plan"]
        lines.append(f"{r['layer']:<52} {r['crs']:>6} {r['mfma_us']:>8.2f} {r['valu_us']:>8.2f} {r['valu_us'] / r['mfma_us']:>9.2f}  "
                     f"{FAMILY[p[0]]} v{p[1]} tile {p[2]}{LOADER.get(p[3], ''):<3}   {r['mfma_parity_ok'] and r['valu_parity_ok']}")
    _write("short_reductions_mfma_vs_valu.txt", lines)


if __name__ == "__main__":
    one = {"traffic": traffic, "counters": counters, "stats": stats, "split_c": split_c, "paper_shapes": paper_shapes,
           "short_reductions": short_reductions}
    if len(sys.argv) >= 3 and sys.argv[1] in ("holdout", "sweep"):
        (holdout if sys.argv[1] == "holdout" else sweep)(sys.argv[2:])
        sys.exit(0)
    if len(sys.argv) != 3 or sys.argv[1] not in tuple(one) + ("commands",):
        sys.exit(__doc__)
    if sys.argv[1] == "commands":     # the counter runs of one layer tag[=shape], one per line
        tag, _, shape = sys.argv[2].partition("=")
        for which in PASSES:
            print(command(tag, shape or None, which))
    else:
        one[sys.argv[1]](sys.argv[2])
