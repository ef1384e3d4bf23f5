"""Builds libconvfwd.so (HIP kernels for gfx950 + the C-ABI) in-tree with hipcc.

Usage: python -m paper_2103_16234_amd.build [--force] [-j N]
The tap-family kernel source is compiled once per (filter size, tile shape) so the
translation units build in parallel; objects are cached under csrc/_build by source mtime.
"""
from __future__ import annotations

import argparse
import concurrent.futures
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libconvfwd.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops is switched off on purpose: packed fp32 forms are not used on this target pool.
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

COMMON += os.environ.get("CONVFWD_EXTRA_HIPCC_FLAGS", "").split()

TAP_SIZES = (1, 3, 5)   # every tile shape; the other filter sizes are read from TAP_EXTRA_SIZES in conv_internal.h


def _num_tap_variants() -> int:
    text = open(os.path.join(CSRC, "conv_internal.h")).read()
    body = re.search(r"kTapVariants\[\]\s*=\s*\{(.*?)\n\};", text, re.S).group(1)
    return len(re.findall(r"^\s*\{", body, re.M))


def _extra_tap_units():
    """(R, S, variant) triples of the tap kernel's other filter sizes, from the two macros that also declare them."""
    text = open(os.path.join(CSRC, "conv_internal.h")).read().replace("\\\n", " ")
    variants = re.search(r"#define TAP_EXTRA_VARIANTS\(X, r, s\)(.*)", text).group(1)
    variants = [int(v) for v in re.findall(r"X\(r, s, (\d+)\)", variants)]
    sizes = re.search(r"#define TAP_EXTRA_SIZES\(X\)(.*)", text).group(1)
    sizes = [(int(r), int(s)) for r, s in re.findall(r"TAP_EXTRA_VARIANTS\(X, (\d+), (\d+)\)", sizes)]
    return [(r, s, v) for r, s in sizes for v in variants]


def _jobs():
    """(object path, source path, extra flags) for every translation unit."""
    jobs = [(os.path.join(OBJ, "convfwd_api.o"), os.path.join(CSRC, "convfwd_api.cpp"), ["-x", "hip"]),
            (os.path.join(OBJ, "generic.o"), os.path.join(CSRC, "generic.hip"), []),
            (os.path.join(OBJ, "pointwise.o"), os.path.join(CSRC, "pointwise_mfma.hip"), []),
            (os.path.join(OBJ, "pointwise_panel.o"), os.path.join(CSRC, "pointwise_panel.hip"), []),
            (os.path.join(OBJ, "two_stage.o"), os.path.join(CSRC, "two_stage.hip"), [])]
    jobs = [j for j in jobs if os.path.exists(j[1])]
    for r in TAP_SIZES:
        for v in range(_num_tap_variants()):
            jobs.append((os.path.join(OBJ, f"tap_{r}x{r}_v{v}.o"), os.path.join(CSRC, "tap_mfma.hip"),
                         [f"-DTAP_R={r}", f"-DTAP_S={r}", f"-DTAP_VARIANT={v}"]))
    for r, s, v in _extra_tap_units():
        jobs.append((os.path.join(OBJ, f"tap_{r}x{s}_v{v}.o"), os.path.join(CSRC, "tap_mfma.hip"),
                     [f"-DTAP_R={r}", f"-DTAP_S={s}", f"-DTAP_VARIANT={v}"]))
    return jobs


def _newest_dep() -> float:
    """What every translation unit depends on: the headers and this script (its own source comes on top)."""
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps += [os.path.join(HERE, "..", "include", "convfwd.h"), os.path.abspath(__file__)]
    return max(os.path.getmtime(d) for d in deps)


def _compile(job, force, stamp):
    obj, src, extra = job
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= max(stamp, os.path.getmtime(src)):
        return obj, 0, ""
    cmd = [HIPCC] + COMMON + extra + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return obj, r.returncode, (r.stdout + r.stderr).strip()


def build(force: bool = False, jobs: int = 0, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    stamp = _newest_dep()
    work = _jobs()
    jobs = jobs or min(8, os.cpu_count() or 1)
    objs = []
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        for obj, rc, out in pool.map(lambda j: _compile(j, force, stamp), work):
            if out and (verbose or rc):
                print(out, file=sys.stderr)
            if rc:
                raise RuntimeError(f"hipcc failed for {obj}")
            objs.append(obj)
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(o) for o in objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("-j", type=int, default=0)
    ap.add_argument("-v", action="store_true")
    ns = ap.parse_args()
    print(build(ns.force, ns.j, ns.v))
