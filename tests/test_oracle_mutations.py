"""The pins of the oracle catch planted mistakes (CPU only).

Each case copies oracle/ to a temporary directory, plants one plausible mistake in conv_ref.c there - a flipped filter,
swapped paddings, a transposed filter index, swapped K and C, a dropped tap, an off-by-one bound, a missing fabs, a wrong
padding passed on - and runs tests/test_oracle_pins.py in a fresh interpreter that imports that copy: the run must fail.
The unchanged copy must pass, so a failure is the mistake's and not the harness's.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = {
    "filter_flipped_along_r": ("int h = p + r - j->pad_h;", "int h = p + (j->R - 1 - r) - j->pad_h;"),
    "filter_flipped_along_s": ("int v = q + s - j->pad_w;", "int v = q + (j->S - 1 - s) - j->pad_w;"),
    "paddings_swapped": ("int v = q + s - j->pad_w;", "int v = q + s - j->pad_h;"),
    "filter_index_transposed": ("(((size_t)k * j->C + c) * j->R + r) * j->S + s", "(((size_t)k * j->C + c) * j->S + s) * j->R + r"),
    "k_and_c_swapped": ("(((size_t)k * j->C + c) * j->R", "(((size_t)c * j->K + k) * j->R"),
    "last_tap_dropped": ("for (int s = 0; s < j->S; ++s)", "for (int s = 0; s < j->S - (j->S > 1); ++s)"),
    "row_bound_off_by_one": ("h >= j->H ||", "h > j->H ||"),
    "fabs_missing": ("acc_abs += fabs(prod);", "acc_abs += prod;"),
    "input_rows_and_columns_swapped": ("* j->H + h) * j->W + v;", "* j->W + v) * j->H + h;"),
}


def _run_pins(tmp_path, text):
    copy = tmp_path / "oracle"
    copy.mkdir()
    for name in ("__init__.py", "conv_ref.py"):
        shutil.copy(os.path.join(ROOT, "oracle", name), copy / name)
    (copy / "conv_ref.c").write_text(text)
    env = dict(os.environ, PYTHONPATH=os.pathsep.join([str(tmp_path), ROOT]))
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-q", "-x",
                           "-p", "no:cacheprovider"], cwd=str(tmp_path), env=env, capture_output=True, text=True, timeout=300)


def _source():
    return open(os.path.join(ROOT, "oracle", "conv_ref.c")).read()


def test_the_unchanged_copy_passes_its_pins(tmp_path):
    r = _run_pins(tmp_path, _source())
    assert r.returncode == 0, r.stdout[-2000:]
    assert str(tmp_path) in subprocess.run(
        [sys.executable, "-c", "import oracle; print(oracle.__file__)"], cwd=str(tmp_path),
        env=dict(os.environ, PYTHONPATH=os.pathsep.join([str(tmp_path), ROOT])), capture_output=True, text=True).stdout


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_a_planted_mistake_fails_the_pins(tmp_path, name):
    old, new = MUTATIONS[name]
    src = _source()
    assert src.count(old) >= 1, f"the line this mutation changes is gone from conv_ref.c: {old}"
    r = _run_pins(tmp_path, src.replace(old, new))
    assert r.returncode != 0, f"the pins did not notice: {name}"
    assert "failed" in r.stdout or "error" in r.stdout.lower()
