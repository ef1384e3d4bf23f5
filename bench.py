#!/usr/bin/env python3
"""Benchmark of the stride-1 forward convolution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config I | --shape N,C,H,W,K,R,S,pad_h,pad_w]
                    [--no-layers] [--no-cpu] [--no-probes]

A step is one conv_fwd call (plan, halo/filter staging, MAC loop, store: the whole hot path) on one
batch of seeded synthetic input that already sits in HBM. The step rotates through enough
(x, w, y) buffer sets to exceed the 256 MB Infinity Cache, so the HBM figures are not cache hits.
Prints ONE JSON line: the headline layer at top level (`config.workload`; by default the largest of the five
benchmark layers, the 3x3 layer with 512 channels at batch 32), plus `layers` with the same measurement for all
five benchmark layers - each with the library's measured mapping and with the cost model's own pick -,
`roofline` for the headline layer's kernel and `cpu_baseline` (the CPU oracle timed on this host on a bounded
sample of the same layer).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

PEAK_FP32_TFLOPS = 157.3   # MI355X dense fp32 (vector packed and matrix), published
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E, published
# Which roofline binds each layer (arithmetic intensity against the 19.7 FLOP/B machine balance; the 1x1
# layer sits near the balance point and is treated as HBM-bound, the tiny first layer is launch-bound).
BOUND = {1: "hbm", 2: "hbm", 3: "mfma", 4: "mfma", 5: "mfma"}
ROOT = os.path.dirname(os.path.abspath(__file__))
# Offline counter readings: bytes per launch that the L2s exchanged with the fabric (Infinity Cache / HBM), from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by what the same counters read for a plain device
# copy of known size. `python -m paper_2103_16234_amd.profiling traffic` writes the table together with the summary
# under profiles/; an entry is only reported while the layer still runs the mapping it was measured with.
TRAFFIC_TABLE = os.path.join(ROOT, "paper_2103_16234_amd", "measured_traffic.json")
KERNEL_NAMES = {0: "conv_generic", 1: "conv_tap_mfma", 2: "conv_pointwise_mfma", 3: "conv_pointwise_panel"}


def measured_traffic(shape, plan):
    """HBM-side bytes per launch from the offline counter table, or None (not measured, or measured with another mapping)."""
    try:
        table = json.load(open(TRAFFIC_TABLE))
    except (OSError, ValueError):
        return None
    rec = table.get("layers", {}).get(",".join(str(d) for d in shape.dims))
    if not rec:
        return None
    if [plan.kernel, plan.variant, plan.tile_pix, plan.loader, plan.order] != rec.get("plan"):
        return None
    return int(rec["fetch_bytes"] + rec["write_bytes"])


def _fail(msg: str, code: int = 2):
    print(msg, file=sys.stderr)
    sys.exit(code)


class Layer:
    """One benchmark layer with rotating device buffers."""

    def __init__(self, index, torch, binding, inputs, min_bytes=600e6, max_sets=2048):
        self.index = index if isinstance(index, int) else None   # a benchmark layer number, or a shape record
        self.shape = inputs.config(index) if isinstance(index, int) else index
        self.torch = torch
        self.lib = binding.load_library()
        x, w = inputs.make_inputs(self.shape)
        self.x_host, self.w_host = x, w
        per_set = self.shape.algorithmic_bytes
        self.sets = int(min(max_sets, max(2, -(-int(min_bytes) // per_set))))
        xd = torch.from_numpy(x).cuda()
        wd = torch.from_numpy(w).cuda()
        self.x = xd.unsqueeze(0).repeat(self.sets, 1, 1, 1, 1)
        self.w = wd.unsqueeze(0).repeat(self.sets, 1, 1, 1, 1)
        self.y = torch.empty((self.sets,) + self.shape.y_shape, device="cuda", dtype=torch.float32)
        self.args = [(ctypes.c_void_p(self.x[i].data_ptr()), ctypes.c_void_p(self.w[i].data_ptr()),
                      ctypes.c_void_p(self.y[i].data_ptr())) for i in range(self.sets)]
        self.dims = tuple(self.shape.dims)
        self.plan = binding.conv_fwd_plan(*self.dims)
        self.calls = 0
        self.request = None

    def step(self):
        xa, wa, ya = self.args[self.calls % self.sets]
        self.calls += 1
        if self.request is not None:
            rc = self.lib.conv_fwd_planned(xa, wa, ya, *self.dims, ctypes.byref(self.request), None)
        else:
            rc = self.lib.conv_fwd(xa, wa, ya, *self.dims)
        if rc != 0:
            raise RuntimeError(f"conv_fwd failed with code {rc}")

    def use_plan(self, plan):
        """Later steps launch the mapping `plan` names (conv_fwd_planned) instead of the library's default; None: default."""
        if plan is None:
            self.request = None
            return
        from paper_2103_16234_amd import binding
        req = binding.ConvPlan()
        req.kernel, req.variant, req.tile_pix, req.loader = plan.kernel, plan.variant, plan.tile_pix, plan.loader
        req.order, req.k_group = plan.order, plan.k_group
        self.request = req

    def measure(self, steps, warmup):
        """Wall clock and HIP-event time over exactly `steps` launches (after `warmup` untimed ones)."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(steps):
            self.step()
        ev1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        event_ms = ev0.elapsed_time(ev1) / steps
        return wall_ms, event_ms

    def single_launches(self, n=25):
        """Every launch between an event pair of its own (the paper's protocol, Section 4: the mean of nine runs per
        configuration): min / median / mean of n launches. Each figure includes the launch gap a lone launch sees."""
        torch = self.torch
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for _ in range(5):
            self.step()
        torch.cuda.synchronize()
        for e0, e1 in pairs:
            e0.record()
            self.step()
            e1.record()
        torch.cuda.synchronize()
        us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in pairs)
        return {"n": n, "min": us[0], "median": us[n // 2], "mean": sum(us) / n}

    def report(self, wall_ms, event_ms, steps):
        s = self.shape
        t = event_ms * 1e-3
        gflops = s.flops / t / 1e9
        gbs = s.algorithmic_bytes / t / 1e9
        bound = self.bound()
        return {
            "layer": s.name, "dims": {"N": s.N, "C": s.C, "H": s.H, "W": s.W, "K": s.K, "R": s.R, "S": s.S,
                                      "pad": s.pad_h},
            "steps": steps, "ms_per_step_wall": wall_ms, "kernel_us": event_ms * 1e3,
            "gflops": gflops, "gbs": gbs,
            "frac_fp32_peak": gflops / (PEAK_FP32_TFLOPS * 1e3), "frac_hbm_peak": gbs / PEAK_HBM_GBS,
            "bound": bound, "buffer_sets": self.sets,
            "plan": {k: getattr(self.plan, k) for k in ("kernel", "variant", "tile_k", "tile_pix", "chunk_c",
                                                         "x_vec", "w_vec", "grid", "block", "lds_bytes", "loader", "order")},
        }

    def bound(self):
        """The benchmark layers carry their stated bound; any other shape takes the slower of its two roofline times."""
        if self.index is not None:
            return BOUND[self.index]
        s = self.shape
        return "hbm" if s.algorithmic_bytes / PEAK_HBM_GBS / 1e9 > s.flops / PEAK_FP32_TFLOPS / 1e12 else "mfma"

    def roofline(self, event_ms):
        s = self.shape
        t = event_ms * 1e-3
        bound = self.bound()
        if bound == "hbm":
            achieved, peak, unit = s.algorithmic_bytes / t / 1e9, PEAK_HBM_GBS, "GB/s"
        else:
            achieved, peak, unit = s.flops / t / 1e12, PEAK_FP32_TFLOPS, "TFLOP/s"
        return {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                "traffic": measured_traffic(s, self.plan), "traffic_source": "offline rocprofv3 FETCH_SIZE + WRITE_SIZE "
                "readings (profiles/conv_kernels_hbm_traffic.txt), not measured in this run",
                "kernel": KERNEL_NAMES.get(self.plan.kernel, "?"),
                "kernel_us": event_ms * 1e3, "algorithmic_bytes": s.algorithmic_bytes, "algorithmic_flops": s.flops}

    def parity_sample(self, oracle, npts=512):
        """Spot check of the timed configuration against the oracle on random output elements."""
        torch = self.torch
        s = self.shape
        rng = np.random.default_rng(7)
        coords = np.stack([rng.integers(0, d, npts) for d in s.y_shape], axis=1).astype(np.int32)
        self.calls = 0
        self.step()
        torch.cuda.synchronize()
        y = self.y[0].cpu().numpy()
        y_ref, ya_ref = oracle.conv_ref_points(self.x_host, self.w_host, s.pad_h, s.pad_w, coords)
        ok, worst = oracle.within_tolerance(y[tuple(coords.T)], y_ref, ya_ref)
        return {"points": npts, "ok": ok, "worst_ratio": worst}


def probes(torch, binding):
    """What this GPU attains, measured with the library's two micro-probes: fp32 MFMA rate and dwordx4 copy bandwidth."""
    lib = binding.load_library()
    sink = torch.zeros(1, device="cuda")
    src = torch.ones(64 * 1024 * 1024, device="cuda")      # 256 MiB each way: past the Infinity Cache
    dst = torch.empty_like(src)
    nbytes = src.numel() * 4
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out = {}
    flops = lib.conv_probe_mfma(2000, sink.data_ptr())
    assert flops > 0
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        lib.conv_probe_mfma(2000, sink.data_ptr())
    e1.record()
    torch.cuda.synchronize()
    out["mfma_fp32_tflops"] = 5 * flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    assert lib.conv_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes) == 0
    torch.cuda.synchronize()
    e0.record()
    for _ in range(10):
        lib.conv_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes)
    e1.record()
    torch.cuda.synchronize()
    out["copy_read_plus_write_gbs"] = 10 * 2 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    assert bool((dst[:: 1 << 20] == 1).all())
    # What one launch costs when the kernel has nothing to do (a 16-byte copy by one work-group), back to back on the
    # library's stream from this same Python loop: the floor under every figure of the batch-1 layers.
    for _ in range(50):
        lib.conv_probe_copy(src.data_ptr(), dst.data_ptr(), 16)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(2000):
        lib.conv_probe_copy(src.data_ptr(), dst.data_ptr(), 16)
    e1.record()
    torch.cuda.synchronize()
    out["empty_launch_us"] = e0.elapsed_time(e1) / 2000 * 1e3
    return out


def cpu_baseline(oracle, inputs, shape, budget_macs=4e9, others=()):
    """The oracle as it stands, on this host's cores, on the whole layer or on its first images; plus one
    single-threaded pass over (a bounded sample of) each layer in `others`."""
    def timed(s, threads, seconds):
        x, w = inputs.make_inputs(s)
        macs_per_image = s.flops / 2 / s.N
        n = int(max(1, min(s.N, budget_macs // macs_per_image)))
        t0 = time.perf_counter()
        oracle.conv_ref(x[:n], w, s.pad_h, s.pad_w, nthreads=threads)
        first = time.perf_counter() - t0
        reps = int(max(1, min(1000, seconds / max(first, 1e-4))))
        t0 = time.perf_counter()
        for _ in range(reps):
            oracle.conv_ref(x[:n], w, s.pad_h, s.pad_w, nthreads=threads)
        dt = (time.perf_counter() - t0) / reps
        return 2 * macs_per_image * n / dt / 1e9, f"{s.name}: images 0..{n - 1} of {s.N}, all {s.K} filters, {reps} pass(es), {dt:.3f} s per pass"

    x, w = inputs.make_inputs(shape)
    oracle.conv_ref(x[:1, :, :4, :4], w[:1], shape.pad_h, shape.pad_w, nthreads=1)   # load the library
    # threads the oracle runs with: the host's cores, at most 16 (one GPU's share of the cores of a multi-GPU host)
    cores = min(os.cpu_count() or 1, 16)
    value, sample = timed(shape, cores, 10.0)                  # about ten seconds of CPU work
    out = {"value": value, "unit": "GFLOP/s", "cores": cores, "kind": "oracle", "sample": sample}
    single = []
    for s in others:                                           # about two seconds each
        v, smp = timed(s, 1, 2.0)
        single.append({"value": v, "unit": "GFLOP/s", "cores": 1, "sample": smp})
    if single:
        out["single_thread"] = single
    return out


# The shapes whose kernel times the paper prints (Tables 3-5: H - N - filter - K - C), with its own stage-1 (+ stage-2)
# time and the best vendor-library time on its GPU (NVIDIA V100, CUDA 9.2), in microseconds: context, not targets.
PAPER_SHAPES = (
    ("1x1 A", (1, 832, 7, 7, 256, 1, 1, 0, 0), 58.56, 107.29),
    ("1x1 B", (1, 256, 14, 14, 1024, 1, 1, 0, 0), 73.86, 45.23),
    ("1x1 C", (1, 64, 27, 27, 256, 1, 1, 0, 0), 22.53, 19.20),
    ("3x3 A", (1, 192, 7, 7, 384, 3, 3, 1, 1), 57.79, 105.63),
    ("3x3 B", (1, 384, 13, 13, 384, 3, 3, 1, 1), 466.68, 232.35),
    ("5x5 A", (1, 48, 7, 7, 128, 5, 5, 2, 2), 22.50, 74.80),
    ("5x5 B", (8, 48, 7, 7, 128, 5, 5, 2, 2), 116.60, 76.58),
)


def paper_shapes(torch, binding, inputs, oracle):
    """Fused kernels (conv_fwd) against the paper's own two-stage scheme (conv_fwd_two_stage) on the paper's shapes."""
    lib = binding.load_library()
    rows = []
    for label, dims, paper_us, vendor_us in PAPER_SHAPES:
        shape = inputs.ConvShape(label, *dims, "u01", "he", 77, 78)
        x, w = inputs.make_inputs(shape)
        sets = 64
        xd = torch.from_numpy(x).cuda().unsqueeze(0).repeat(sets, 1, 1, 1, 1)
        wd = torch.from_numpy(w).cuda().unsqueeze(0).repeat(sets, 1, 1, 1, 1)
        yd = torch.empty((sets,) + shape.y_shape, device="cuda")
        need = binding.conv_two_stage_workspace_bytes(*dims)
        ws = torch.empty(max(need // 4, 1), device="cuda")

        def fused(i):
            return lib.conv_fwd(xd[i].data_ptr(), wd[i].data_ptr(), yd[i].data_ptr(), *dims)

        def staged(i):
            return lib.conv_fwd_two_stage(xd[i].data_ptr(), wd[i].data_ptr(), yd[i].data_ptr(), ws.data_ptr(), need, *dims)

        rec = {"shape": label, "dims": dict(zip("N C H W K R S pad_h pad_w".split(), dims)),
               "paper_two_stage_us_v100": paper_us, "paper_best_vendor_us_v100": vendor_us}
        y_ref, ya_ref = oracle.conv_ref(x, w, shape.pad_h, shape.pad_w)
        for name, fn in (("fused_us", fused), ("two_stage_us", staged)):
            for i in range(10):
                assert fn(i % sets) == 0
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(500):
                fn(i % sets)
            e1.record()
            torch.cuda.synchronize()
            rec[name] = e0.elapsed_time(e1) / 500 * 1e3
            assert fn(0) == 0
            torch.cuda.synchronize()
            rec[name.replace("_us", "_parity_ok")] = oracle.within_tolerance(yd[0].cpu().numpy(), y_ref, ya_ref)[0]
        plan = binding.conv_fwd_plan(*dims)
        rec["fused_plan"] = {"kernel": plan.kernel, "variant": plan.variant, "grid": plan.grid, "block": plan.block}
        rows.append(rec)
    return rows


def sweep(torch, binding, inputs, oracle, only=None, find=False):
    """Second workload: every shape of the synthetic sweep grid, timed like the layers and spot-checked against the oracle."""
    rows = []
    flush = torch.empty(128 * 1024 * 1024, device="cuda") if find else None   # 512 MiB: twice the Infinity Cache
    for shape in inputs.sweep_shapes():
        if only and only not in shape.name:
            continue
        layer = Layer(shape, torch, binding, inputs, min_bytes=600e6, max_sets=256)
        _, ev = layer.measure(3, 2)
        k = int(max(10, min(1000, 0.05 / max(ev * 1e-3, 1e-7))))
        w_ms, e_ms = layer.measure(k, 3)
        roof = layer.roofline(e_ms)
        par = layer.parity_sample(oracle, 128)
        p = layer.plan
        rec = {"shape": shape.name, "kernel_us": e_ms * 1e3, "tflops": shape.flops / e_ms / 1e9,
               "gbs": shape.algorithmic_bytes / e_ms / 1e6, "bound": roof["bound"], "frac": roof["frac"],
               "plan": [p.kernel, p.variant, p.tile_pix, p.grid, p.block, p.loader], "parity_ok": par["ok"]}
        if find:
            # measured choice of the mapping (conv_fwd_find), then the same rotating-buffer timing with it
            _, fp, _ = binding.conv_fwd_find(layer.x[0], layer.w[0], shape.pad_h, shape.pad_w, y=layer.y[0], flush=flush)
            _, f_ms = layer.measure(k, 3)
            fpar = layer.parity_sample(oracle, 128)
            # once more each, the default now by request: whichever mapping is timed right after the search's burst of
            # launches finds the clocks up, which is worth up to 20 % on layers of a few microseconds
            layer.use_plan(p)
            e_ms = min(e_ms, layer.measure(k, 3)[1])
            layer.use_plan(None)
            f_ms = min(f_ms, layer.measure(k, 3)[1])
            roof = layer.roofline(e_ms)
            rec.update({"kernel_us": e_ms * 1e3, "tflops": shape.flops / e_ms / 1e9, "gbs": shape.algorithmic_bytes / e_ms / 1e6,
                        "frac": roof["frac"]})
            rec.update({"found_us": f_ms * 1e3, "found_plan": [fp.kernel, fp.variant, fp.tile_pix, fp.grid, fp.block, fp.loader],
                        "found_frac": layer.roofline(f_ms)["frac"], "found_parity_ok": fpar["ok"]})
        rows.append(rec)
        print(f"sweep {shape.name}: {e_ms * 1e3:.1f} us {roof['bound']} {roof['frac']:.3f} parity {par['ok']}",
              file=sys.stderr, flush=True)
        del layer
        torch.cuda.empty_cache()
    return rows


def holdout(torch, binding, inputs, oracle, seed, count=40):
    """Planner check on layers it was not fitted on: `count` random shapes inside the paper's ranges but off the sweep
    grid (other batch sizes, channel counts and map sizes), each timed with the default mapping and with the one
    conv_fwd_find measures to be fastest."""
    import random
    rng = random.Random(seed)
    flush = torch.empty(128 * 1024 * 1024, device="cuda")
    shapes = []
    while len(shapes) < count:
        f = rng.choice([1, 3, 3, 5])
        n = rng.choice([1, 2, 4, 16, 64])
        h = rng.choice([7, 10, 14, 17, 20, 28, 35, 40, 56, 80, 112])
        c = rng.choice([16, 24, 48, 80, 128, 160, 320, 448, 640])
        k = rng.choice([24, 48, 96, 160, 256, 320, 512, 768])
        if (f == 5 and c > 128) or n * c * h * h > 2 ** 24 or n * k * h * h > 2 ** 24:
            continue
        shapes.append(inputs.ConvShape(f"holdout_{f}x{f}_n{n}_c{c}_{h}_k{k}", n, c, h, h, k, f, f, f // 2, f // 2, "u01", "he",
                                       5000 + len(shapes), 6000 + len(shapes)))
    rows = []
    for shape in shapes:
        layer = Layer(shape, torch, binding, inputs, min_bytes=400e6, max_sets=32)
        _, ev = layer.measure(10, 5)
        k = int(max(20, min(500, 0.02 / max(ev * 1e-3, 1e-7))))
        layer.measure(k, 3)                                   # clocks and caches settle: the second run counts
        _, d_ms = layer.measure(k, 3)
        _, fp, _ = binding.conv_fwd_find(layer.x[0], layer.w[0], shape.pad_h, shape.pad_w, y=layer.y[0], flush=flush)
        _, f_ms = layer.measure(k, 3)
        par = layer.parity_sample(oracle, 64)
        p = layer.plan
        # once more each, the default now by request (see sweep): the faster of a mapping's two runs counts
        layer.use_plan(p)
        d_ms = min(d_ms, layer.measure(k, 3)[1])
        layer.use_plan(None)
        f_ms = min(f_ms, layer.measure(k, 3)[1])
        rows.append({"shape": shape.name, "default_us": d_ms * 1e3, "found_us": f_ms * 1e3, "frac": layer.roofline(d_ms)["frac"],
                     "default_plan": [p.kernel, p.variant, p.tile_pix, p.grid, p.block, p.loader],
                     "found_plan": [fp.kernel, fp.variant, fp.tile_pix, fp.grid, fp.block, fp.loader], "found_parity_ok": par["ok"]})
        print(f"holdout {shape.name}: default {d_ms * 1e3:.1f} us, found {f_ms * 1e3:.1f} us, parity {par['ok']}", file=sys.stderr,
              flush=True)
        del layer
        torch.cuda.empty_cache()
    ratios = [r["default_us"] / min(r["default_us"], r["found_us"]) for r in rows]
    return {"seed": seed, "layers": rows, "default_over_found_geomean": float(np.exp(np.mean(np.log(ratios)))),
            "default_over_found_worst": max(ratios)}


def split_c_layers(torch, binding, inputs, oracle):
    """Channel splitting across work-groups (conv_fwd_split_c) against the single-kernel default, on every layer of the
    sweep grid and of the paper's profiled shapes for which the splitting planner asks for more than one share."""
    lib = binding.load_library()
    shapes = list(inputs.sweep_shapes()) + [inputs.ConvShape(label, *dims, "u01", "he", 77, 78)
                                            for label, dims, _, _ in PAPER_SHAPES]
    rows = []
    for shape in shapes:
        sp = binding.conv_fwd_plan_split_c(*shape.dims)
        if sp.c_splits <= 1:
            continue
        layer = Layer(shape, torch, binding, inputs, min_bytes=600e6, max_sets=256)
        ws = torch.empty(sp.workspace_bytes // 4, device="cuda")

        def split_step():
            xa, wa, ya = layer.args[layer.calls % layer.sets]
            layer.calls += 1
            rc = lib.conv_fwd_split_c(xa, wa, None, ya, ctypes.c_void_p(ws.data_ptr()), sp.workspace_bytes, *layer.dims, 0,
                                      None, None)
            if rc != 0:
                raise RuntimeError(f"conv_fwd_split_c failed with code {rc}")

        k = 400
        _, d_ms = layer.measure(k, 10)
        default_step, layer.step = layer.step, split_step
        _, s_ms = layer.measure(k, 10)
        par = layer.parity_sample(oracle, 128)
        layer.step = default_step
        p = layer.plan
        rows.append({"shape": shape.name, "dims": list(shape.dims), "default_us": d_ms * 1e3, "split_us": s_ms * 1e3,
                     "default_plan": [p.kernel, p.variant, p.tile_pix, p.grid, p.block, p.loader],
                     "split_plan": [sp.kernel, sp.variant, sp.tile_pix, sp.grid, sp.block, sp.loader], "c_splits": sp.c_splits,
                     "workspace_bytes": sp.workspace_bytes, "split_parity_ok": par["ok"]})
        print(f"split-c {shape.name}: default {d_ms * 1e3:.1f} us, {sp.c_splits} shares {s_ms * 1e3:.1f} us, parity {par['ok']}",
              file=sys.stderr, flush=True)
        del layer, ws
        torch.cuda.empty_cache()
    return rows


def layer_record(layer, torch, binding, oracle, measured, warmup, auto_steps):
    """One entry of `layers`: the planner's mapping of the layer (the benchmark layers go through the same cost model and
    rules as every other shape: the library keeps no table of measured mappings)."""
    k = auto_steps(layer)
    w_ms, e_ms = layer.measure(k, warmup)
    rec = layer.report(w_ms, e_ms, k)
    rec["parity"] = layer.parity_sample(oracle, 256)
    rec["single_launch_us"] = layer.single_launches()
    rec["frac_of_measured_mfma"] = rec["gflops"] / 1e3 / measured["mfma_fp32_tflops"]
    rec["frac_of_measured_copy_bw"] = rec["gbs"] / measured["copy_read_plus_write_gbs"]
    rec["roofline"] = layer.roofline(e_ms)
    return rec


# Layers with a short reduction (C*R*S of 27 ... 400): is the matrix unit the right tool there?
SHORT_REDUCTIONS = (
    ("cfg1: 3x3 C16 14x14 K16 N1 (C*R*S = 144)", (1, 16, 14, 14, 16, 3, 3, 1, 1)),
    ("first layer: 3x3 C3 224x224 K64 N1 (C*R*S = 27)", (1, 3, 224, 224, 64, 3, 3, 1, 1)),
    ("first layer: 3x3 C3 224x224 K64 N8 (C*R*S = 27)", (8, 3, 224, 224, 64, 3, 3, 1, 1)),
    ("3x3 C16 224x224 K16 N1 (C*R*S = 144)", (1, 16, 224, 224, 16, 3, 3, 1, 1)),
    ("3x3 C16 56x56 K16 N8 (C*R*S = 144)", (8, 16, 56, 56, 16, 3, 3, 1, 1)),
    ("5x5 C16 28x28 K32 N1 (C*R*S = 400)", (1, 16, 28, 28, 32, 5, 5, 2, 2)),
)


def short_reductions(torch, binding, inputs, oracle):
    """The library's two ways of multiplying on layers with a short reduction: the default mapping (fp32 MFMA in the
    specialised kernels) against the generic kernel (one output per thread, plain vector fp32 FMA)."""
    rows = []
    for name, dims in SHORT_REDUCTIONS:
        layer = Layer(inputs.ConvShape(name, *dims, "u01", "he", 31, 32), torch, binding, inputs, max_sets=256)
        rec = {"layer": name, "dims": list(dims), "crs": dims[1] * dims[5] * dims[6],
               "default_plan": [layer.plan.kernel, layer.plan.variant, layer.plan.tile_pix, layer.plan.loader]}
        for label, plan in (("mfma", None), ("valu", binding.ConvPlan())):      # a zeroed request names the generic kernel
            layer.use_plan(plan)
            _, e_ms = layer.measure(500, 20)
            rec[label + "_us"] = e_ms * 1e3
            rec[label + "_parity_ok"] = layer.parity_sample(oracle, 128)["ok"]
        rows.append(rec)
        del layer
        torch.cuda.empty_cache()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed launches of the headline layer (0 = auto: about 0.25 s)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=5,
                    help="headline layer, 1..5 (default 5: the largest one, 3x3 with 512 channels at batch 32)")
    ap.add_argument("--shape", default=None, metavar="N,C,H,W,K,R,S,PAD_H,PAD_W",
                    help="headline layer given by its nine dimensions instead of --config (counter runs on other layers)")
    ap.add_argument("--no-layers", action="store_true", help="skip the per-layer table")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-probes", action="store_true", help="skip the two micro-probes of attainable peaks")
    ap.add_argument("--paper-shapes", action="store_true",
                    help="also time the fused kernels and the paper's two-stage scheme on the shapes the paper profiles")
    ap.add_argument("--sweep", nargs="?", const="", default=None, metavar="SUBSTR",
                    help="also run the synthetic shape sweep (optionally only shapes whose name contains SUBSTR)")
    ap.add_argument("--find", action="store_true",
                    help="with --sweep: also time each layer with the mapping conv_fwd_find measures to be fastest")
    ap.add_argument("--holdout", type=int, default=None, metavar="SEED",
                    help="also compare default and measured-best mappings on 40 random layers off the sweep grid")
    ap.add_argument("--short-reductions", action="store_true",
                    help="also time MFMA against plain vector FMA (the generic kernel) on layers with a short reduction")
    ap.add_argument("--split-c", action="store_true",
                    help="also compare the channel-splitting mode with the default on the layers its planner splits")
    ns = ap.parse_args()
    if ns.gpus != 1:
        _fail("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
    if not 1 <= ns.config <= 5:
        _fail("bench.py: --config must be 1..5")

    import torch
    if not torch.cuda.is_available():
        _fail("bench.py: no GPU visible; the HIP path has no CPU fallback")
    import oracle
    from paper_2103_16234_amd import binding, inputs

    binding.load_library()
    binding.conv_set_stream(torch.cuda.current_stream())
    # A plain 64 MiB device-to-device copy: the known-size kernel the FETCH_SIZE / WRITE_SIZE counters are scaled by.
    calib = torch.ones(16 * 1024 * 1024, device="cuda")
    calib = calib.clone()
    torch.cuda.synchronize()
    del calib

    def auto_steps(layer):
        _, ev = layer.measure(5, 3)
        return int(max(50, min(5000, 0.25 / max(ev * 1e-3, 1e-7))))

    if ns.shape:
        try:
            dims = tuple(int(v) for v in ns.shape.split(","))
            assert len(dims) == 9
        except (ValueError, AssertionError):
            _fail("bench.py: --shape takes nine comma-separated integers")
        head_shape = inputs.ConvShape("shape_" + "_".join(str(d) for d in dims), *dims, "u01", "he", 1100, 2100)
        head = Layer(head_shape, torch, binding, inputs)
    else:
        head = Layer(ns.config, torch, binding, inputs)
    steps = ns.steps or auto_steps(head)
    wall_ms, event_ms = head.measure(steps, ns.warmup)
    parity = head.parity_sample(oracle)
    s = head.shape
    out = {
        "metric": "effective GFLOP/s per conv layer + % of FP32 peak or HBM GB/s roofline",
        "value": s.flops / (wall_ms * 1e-3) / 1e9, "unit": "GFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": ns.warmup, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{s.name}: N={s.N} C={s.C} H={s.H} W={s.W} K={s.K} R={s.R} S={s.S} pad={s.pad_h},{s.pad_w} "
                               f"stride 1, NCHW fp32, {head.sets} rotating buffer sets",
                   "gbs": s.algorithmic_bytes / (wall_ms * 1e-3) / 1e9,
                   "plan": {k: getattr(head.plan, k) for k in ("kernel", "variant", "tile_pix", "grid", "block", "lds_bytes", "loader", "order")}},
        "roofline": head.roofline(event_ms),
        "parity": parity,
    }
    del head
    torch.cuda.empty_cache()
    measured = None
    if not ns.no_probes:
        measured = probes(torch, binding)
        out["probes"] = measured
        roof = out["roofline"]
        roof["frac_of_measured"] = roof["achieved"] / (measured["copy_read_plus_write_gbs"] if roof["bound"] == "hbm"
                                                       else measured["mfma_fp32_tflops"])
        torch.cuda.empty_cache()
    if not ns.no_layers and measured is not None:
        layers = []
        for i in range(1, 6):
            layer = Layer(i, torch, binding, inputs)
            layers.append(layer_record(layer, torch, binding, oracle, measured, ns.warmup, auto_steps))
            del layer
            torch.cuda.empty_cache()
        out["layers"] = layers
        # The 1x1 benchmark layer is launch-bound at batch 1 (its roofline time is below one kernel dispatch): the same layer
        # at larger batches, and an HBM-bound 64 -> 64 channel layer, show what the 1x1 path sustains.
        scaled = []
        for name, dims in (("cfg2 at N=32", (32, 256, 56, 56, 64, 1, 1, 0, 0)), ("cfg2 at N=128", (128, 256, 56, 56, 64, 1, 1, 0, 0)),
                           ("1x1 64->64 channels, 56x56, N=128", (128, 64, 56, 56, 64, 1, 1, 0, 0))):
            layer = Layer(inputs.ConvShape(name, *dims, "u01", "he", 1002, 2002), torch, binding, inputs, max_sets=16)
            k = auto_steps(layer)
            _, e_ms = layer.measure(k, ns.warmup)
            roof = layer.roofline(e_ms)
            scaled.append({"layer": name, "kernel_us": e_ms * 1e3, "tflops": layer.shape.flops / e_ms / 1e9,
                           "gbs": layer.shape.algorithmic_bytes / e_ms / 1e6, "bound": roof["bound"], "frac": roof["frac"],
                           "frac_hbm_peak": layer.shape.algorithmic_bytes / e_ms / 1e6 / PEAK_HBM_GBS,
                           "frac_of_measured_copy_bw": layer.shape.algorithmic_bytes / e_ms / 1e6 / measured["copy_read_plus_write_gbs"],
                           "traffic": roof["traffic"],
                           "parity_ok": layer.parity_sample(oracle, 128)["ok"]})
            del layer
            torch.cuda.empty_cache()
        out["batch_scaled_1x1"] = scaled
    if ns.paper_shapes:
        out["paper_shapes"] = paper_shapes(torch, binding, inputs, oracle)
    if ns.sweep is not None:
        out["sweep"] = sweep(torch, binding, inputs, oracle, ns.sweep, ns.find)
    if ns.holdout is not None:
        out["holdout"] = holdout(torch, binding, inputs, oracle, ns.holdout)
    if ns.split_c:
        out["split_c"] = split_c_layers(torch, binding, inputs, oracle)
    if ns.short_reductions:
        out["short_reductions"] = short_reductions(torch, binding, inputs, oracle)
    if not ns.no_cpu:
        others = [inputs.config(i) for i in range(1, 5)] if not ns.shape and not ns.no_layers else []
        out["cpu_baseline"] = cpu_baseline(oracle, inputs, s, others=others)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
