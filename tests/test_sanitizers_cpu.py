"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host code (CPU only; sanitizers cannot run on the GPU here).

* the oracle (oracle/conv_ref.c) with a C driver that also checks closed forms;
* the planner and argument validation (csrc/convfwd_api.cpp, host pass only sanitized) linked with the kernels' objects
  into an executable that plans every layer of the sweep grid, the benchmark layers and a set of hostile shapes, with
  every host-only entry point and with requests for every tile shape. No device is touched.
"""
import os
import shutil
import subprocess

import pytest

from paper_2103_16234_amd import build as hip_build
from paper_2103_16234_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = tmp_path / "sanitize_oracle"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-ffp-contract=off",
                    "-o", str(exe), os.path.join(NATIVE, "sanitize_oracle.c"), os.path.join(ROOT, "oracle", "conv_ref.c"),
                    "-lpthread", "-lm"], check=True)
    r = subprocess.run([str(exe)], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "0 problems" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


HOSTILE = [
    (1, 64, 3, 7, 16, 3, 3, 0, 5600000), (1, 4, 3, 7, 1, 3, 3, 0, 400000000), (1, 16, 3, 40000, 16, 3, 3, 1, 1),
    (1, 5, 1, 46000, 3, 1, 1, 0, 0), (4095, 8, 256, 256, 3, 3, 3, 1, 1), (1, 1, 1, 1, 1, 1, 1, 0, 0), (1, 3, 1, 2000000, 2, 1, 1, 0, 0),
    (1, 1, 2000000, 1, 2, 3, 1, 1, 0), (2, 7, 5, 5, 9, 7, 7, 3, 3), (1, 2147483647, 1, 1, 1, 1, 1, 0, 0), (1, 4, 8, 8, 4, 9, 9, 0, 0),
    (1, 2147483644, 1, 1, 1, 1, 1, 0, 0), (1, 1073741824, 1, 1, 1, 1, 1, 0, 0), (1, 4, 1, 1, 500000000, 1, 1, 0, 0), (2, 4, 23170, 23170, 1, 1, 1, 0, 0),
    (1, 1, 46340, 46340, 1, 3, 3, 1, 1), (1, 8, 1, 1, 8, 3, 3, 1000000, 1), (1, 1048576, 2, 2, 256, 1, 1, 0, 0), (2047, 1024, 1, 1, 1024, 1, 1, 0, 0),
    (0, 4, 8, 8, 4, 3, 3, 1, 1), (1, 4, 8, 8, 4, 3, 3, -1, 1), (3, 12, 2, 2, 2049, 5, 5, 2, 2), (65536, 16, 2, 2, 16, 1, 1, 0, 0),
]


def test_planner_under_address_and_undefined_sanitizers(tmp_path):
    objects = os.path.join(ROOT, "paper_2103_16234_amd", "csrc", "_build")
    if not os.path.isdir(objects) or not os.path.exists(os.path.join(objects, "generic.o")):
        hip_build.build()
    hipcc = hip_build.HIPCC
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    api = tmp_path / "convfwd_api_san.o"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    subprocess.run([hipcc] + hip_build.COMMON + san + ["-g", "-x", "hip", "-c", os.path.join(ROOT, "paper_2103_16234_amd", "csrc", "convfwd_api.cpp"),
                    "-o", str(api)], check=True, capture_output=True)
    others = [obj for obj, _, _ in hip_build._jobs() if not obj.endswith("convfwd_api.o")]     # the kernels' objects, as built
    driver = tmp_path / "sanitize_host.o"
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-c",
                    os.path.join(NATIVE, "sanitize_host.cpp"), "-o", str(driver)], check=True, capture_output=True)
    exe = tmp_path / "sanitize_host"
    link = subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-g", "-o",
                           str(exe), str(driver), str(api)] + others, capture_output=True, text=True)
    assert link.returncode == 0, link.stderr[-3000:]
    shapes = [s.dims for s in inputs.sweep_shapes()[::3]] + [inputs.config(i).dims for i in range(1, 6)] + HOSTILE
    text = "\n".join(" ".join(str(v) for v in d) for d in shapes) + "\n"
    r = subprocess.run([str(exe)], input=text, env=ENV, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    plans = int(r.stdout.split()[1])
    assert plans > 20 * len(shapes)
    shutil.rmtree(tmp_path, ignore_errors=True)
