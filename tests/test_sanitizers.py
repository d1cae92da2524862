"""Sanitizer leg (CPU only): the host planner and the float64 oracle, compiled with AddressSanitizer and
UndefinedBehaviorSanitizer and driven over seeded random batches by tests/sanitize_driver.cpp (which also checks
the planner's tables and the oracle's values, see its header).  Any invalid access, leak, overflow or failed check
ends the driver with a non-zero status."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc and g++")
def test_planner_and_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    planner = os.path.join(ROOT, "paper_2411_00915_amd", "csrc", "planner.cpp")
    oracle_c = os.path.join(ROOT, "oracle", "lora_oracle.c")
    driver = os.path.join(ROOT, "tests", "sanitize_driver.cpp")
    objs = []
    for cc, src, std in (("g++", planner, "-std=c++17"), ("gcc", oracle_c, "-std=c11"), ("g++", driver, "-std=c++17")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        extra = ["-fopenmp", "-ffp-contract=off"] if src == oracle_c else []
        subprocess.run([cc, "-c", src, "-o", obj, std, "-Wall"] + SAN + extra, check=True)
        objs.append(obj)
    exe = str(tmp_path / "sanitize_driver")
    # the sanitizer runtimes are linked statically: they must come first in the process's library list, which a
    # preloaded library in the environment would otherwise prevent
    subprocess.run(["g++", "-o", exe] + objs + SAN + ["-fopenmp", "-static-libasan", "-static-libubsan"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, f"sanitizer run failed (status {res.returncode}):\n{res.stdout[-2000:]}\n{res.stderr[-6000:]}"
    assert "sanitize_driver: ok" in res.stdout
    assert "runtime error" not in res.stderr and "ERROR: AddressSanitizer" not in res.stderr and \
        "LeakSanitizer" not in res.stderr, res.stderr[-6000:]
