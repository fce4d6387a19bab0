"""Sanitizer passes on the CPU (no GPU): the oracle, and the library itself -- its host code
(launch plan, workspace layout) and its kernels, compiled as host C++ against a small emulation
of workgroups and wavefront builtins -- are built with AddressSanitizer +
UndefinedBehaviorSanitizer into native test programs; the oracle's pin suite is also run
against an UndefinedBehaviorSanitizer build of the shared library.  Sanitizers stay on the
CPU: no instrumented code ever runs on the GPU."""
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


EMU_SOURCES = ["dgs_stream.hip", "dgs_select.hip", "dgs_chain.hip", "dgs_server.hip", "dgs_api.hip"]


def build_emulated_kernels(outdir, seg_tiles=16, group_tiles=64, opt="-O2"):
    """The library's own .hip sources compiled as host C++ against tests/emu (a fiber-based
    emulation of workgroups, wavefront builtins and the few HIP calls used), with ASan + UBSan,
    linked with the oracle and the scenario driver."""
    clang = os.environ.get("DGS_HOST_CLANG", "/opt/rocm/llvm/bin/clang++")
    emu = os.path.join(HERE, "emu")
    csrc = os.path.join(ROOT, "paper_1910_10929_amd", "csrc")
    flags = ["-std=c++17", opt, "-g", f"-I{emu}", f"-DDGS_SEG_TILES={seg_tiles}",
             f"-DDGS_GROUP_TILES={group_tiles}", "-ffp-contract=off",
             "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wno-unknown-attributes",
             "-Wno-unused-function", "-Wno-array-compare"]
    objs, procs = [], []
    for src in EMU_SOURCES:
        o = os.path.join(outdir, src + ".o")
        objs.append(o)
        procs.append(subprocess.Popen([clang, "-x", "c++"] + flags + ["-c", os.path.join(csrc, src), "-o", o]))
    for name in ("emu_core.cpp", "emu_driver.cpp"):
        o = os.path.join(outdir, name + ".o")
        objs.append(o)
        procs.append(subprocess.Popen([clang] + flags + ["-c", os.path.join(emu, name), "-o", o]))
    o = os.path.join(outdir, "oracle.o")
    objs.append(o)
    procs.append(subprocess.Popen([clang.replace("clang++", "clang"), "-std=c99", "-O1", "-g", "-ffp-contract=off",
                                   "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-c",
                                   os.path.join(ROOT, "oracle", "dgs_oracle.c"), "-o", o]))
    for p in procs:
        assert p.wait() == 0, "compiling the emulated kernels failed"
    exe = os.path.join(outdir, "emu_run")
    subprocess.run([clang, "-fsanitize=address,undefined"] + objs + ["-o", exe, "-lm"], check=True)
    return exe


def test_kernels_on_the_cpu_under_asan_ubsan(tmp_path):
    """The HIP kernels and the host code of libdgs, run on the CPU through the C ABI against the
    oracle, bit for bit, with every buffer an exact-size heap block: the streaming pass, the
    selection launch with joins by several workgroups and re-collection after failed
    predictions, the chain kernels, the entry point that allocates nothing, wire form, apply,
    pull_all.  (`emu_run` without arguments runs the long list of scenarios, `emu_run soak
    <seed> <count>` randomised ones, `emu_run rounds` -- built with seg_tiles=256 and
    group_tiles=4096, the library's own sizes -- joins of several rounds per workgroup and the
    trimming of one workgroup's overlong list; this test runs the short list.)"""
    exe = build_emulated_kernels(str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")
    r = subprocess.run([exe, "quick"], capture_output=True, text=True, env=env, timeout=1500)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-6000:]
    assert "all scenarios match the oracle" in r.stdout


def test_oracle_pins_against_ubsan_build():
    env = dict(os.environ, DGS_ORACLE_SANITIZE="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(HERE, "test_oracle_pins.py")],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout
