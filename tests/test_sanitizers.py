"""Sanitizer passes over the CPU-side code (no GPU): the oracle, and the host-only launch
plan of the library, are compiled with AddressSanitizer + UndefinedBehaviorSanitizer into
native test programs that run them over ragged, tiny and benchmark-shaped layouts; the
oracle's pin suite is also run against an UndefinedBehaviorSanitizer build of the shared
library.  Sanitizers stay on the CPU: nothing here touches device code."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
       "-fno-omit-frame-pointer"]


def _build_and_run(tmp_path, compiler, std, sources, name, includes=()):
    exe = str(tmp_path / name)
    cmd = [compiler, std, "-Wall", "-Wextra", "-ffp-contract=off"] + SAN
    cmd += [f"-I{i}" for i in includes] + ["-o", exe] + sources + ["-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, f"{name} failed ({r.returncode}):\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    return r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    out = _build_and_run(tmp_path, "gcc", "-std=c99",
                         [os.path.join(ROOT, "oracle", "dgs_oracle.c"),
                          os.path.join(HERE, "sanitize", "oracle_driver.c")], "oracle_driver")
    assert "oracle sanitizer driver: ok" in out


def test_oracle_pins_against_ubsan_build():
    env = dict(os.environ, DGS_ORACLE_SANITIZE="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(HERE, "test_oracle_pins.py")],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout
