"""ctypes access to the C oracle (`dgs_oracle.c`).

Test infrastructure only: tests, the smoke check and the benchmark's CPU
baseline use it; the product package never does.  Argument marshalling only;
every arithmetic step is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dgs_oracle.c")
_LIB = os.path.join(_HERE, "libdgs_oracle.so")

_c_f32p = ctypes.POINTER(ctypes.c_float)
_c_u32p = ctypes.POINTER(ctypes.c_uint32)
_c_u64p = ctypes.POINTER(ctypes.c_uint64)


# DGS_ORACLE_SANITIZE=1 in the environment: the tests run against a build with the
# undefined-behaviour sanitizer compiled in (any report aborts the process).
_SANITIZE = os.environ.get("DGS_ORACLE_SANITIZE", "") == "1"
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libdgs_oracle_ubsan.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no contraction, no FTZ."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        extra = ["-g", "-fsanitize=undefined", "-fno-sanitize-recover=all"] if _SANITIZE else []
        cmd = ["gcc", "-std=c99", "-O2", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra"] + extra + ["-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.dgs_oracle_k.restype = ctypes.c_uint64
        L.dgs_oracle_k.argtypes = [ctypes.c_double, ctypes.c_uint64]
        L.dgs_oracle_nnz.argtypes = [_c_u64p, ctypes.c_uint32, ctypes.c_double, _c_u64p, _c_u64p]
        L.dgs_oracle_topk.argtypes = [_c_f32p, ctypes.c_uint64, ctypes.c_uint64, _c_u32p]
        L.dgs_oracle_topk_bruteforce.argtypes = [_c_f32p, ctypes.c_uint32, ctypes.c_uint32, _c_u32p]
        L.dgs_oracle_worker_step.argtypes = [_c_f32p, _c_f32p, _c_u64p, ctypes.c_uint32,
                                             ctypes.c_float, ctypes.c_float, ctypes.c_double,
                                             _c_u32p, _c_f32p, _c_u64p]
        L.dgs_oracle_server_push.argtypes = [_c_f32p, _c_f32p, ctypes.c_uint32, ctypes.c_uint64,
                                             _c_u32p, _c_f32p, ctypes.c_uint64]
        L.dgs_oracle_server_pull.argtypes = [_c_f32p, _c_u64p, ctypes.c_uint32, ctypes.c_double,
                                             _c_u32p, _c_f32p, _c_u64p]
        L.dgs_oracle_server_pull_all.argtypes = [_c_f32p, ctypes.c_uint64, _c_u32p, _c_f32p,
                                                 ctypes.c_uint64, _c_u64p]
        L.dgs_oracle_apply_sparse.argtypes = [_c_f32p, ctypes.c_uint64, _c_u32p, _c_f32p,
                                              ctypes.c_uint64, ctypes.c_float]
        L.dgs_oracle_server_push_model.argtypes = [_c_f32p, ctypes.c_uint64, _c_u32p, _c_f32p,
                                                   ctypes.c_uint64]
        L.dgs_oracle_server_pull_sent.argtypes = [_c_f32p, _c_f32p, _c_u64p, ctypes.c_uint32,
                                                  ctypes.c_double, _c_u32p, _c_f32p, _c_u64p]
        L.dgs_oracle_server_pull_all_sent.argtypes = [_c_f32p, _c_f32p, ctypes.c_uint64, _c_u32p, _c_f32p,
                                                      ctypes.c_uint64, _c_u64p]
        _c_u8p = ctypes.POINTER(ctypes.c_uint8)
        L.dgs_oracle_wire_bytes.argtypes = [_c_u64p, ctypes.c_uint32, ctypes.c_double, _c_u64p]
        L.dgs_oracle_encode.argtypes = [_c_u64p, ctypes.c_uint32, ctypes.c_double, _c_u32p, _c_f32p, _c_u8p]
        L.dgs_oracle_decode.argtypes = [_c_u64p, ctypes.c_uint32, ctypes.c_double, _c_u8p, _c_u32p, _c_f32p]
        L.dgs_oracle_wire_bytes16.argtypes = [_c_u64p, ctypes.c_uint32, ctypes.c_double, _c_u64p]
        L.dgs_oracle_encode16.argtypes = [_c_u64p, ctypes.c_uint32, ctypes.c_double, _c_u32p, _c_f32p, _c_u8p]
        L.dgs_oracle_decode16.argtypes = [_c_u64p, ctypes.c_uint32, ctypes.c_double, _c_u8p, _c_u32p, _c_f32p]
        _lib = L
    return _lib


def _f32(a):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(_c_f32p)


def _u32(a):
    assert a.dtype == np.uint32 and a.flags.c_contiguous
    return a.ctypes.data_as(_c_u32p)


def _u64(a):
    assert a.dtype == np.uint64 and a.flags.c_contiguous
    return a.ctypes.data_as(_c_u64p)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def k_of(density: float, n: int) -> int:
    return int(lib().dgs_oracle_k(float(density), int(n)))


def nnz(offsets: np.ndarray, density: float):
    """(k_per_tensor, K)."""
    J = len(offsets) - 1
    kj = np.zeros(J, dtype=np.uint64)
    K = ctypes.c_uint64(0)
    _check(lib().dgs_oracle_nnz(_u64(offsets), J, float(density), _u64(kj), ctypes.byref(K)), "nnz")
    return kj, int(K.value)


def topk(a: np.ndarray, k: int) -> np.ndarray:
    out = np.zeros(k, dtype=np.uint32)
    _check(lib().dgs_oracle_topk(_f32(a), a.size, k, _u32(out)), "topk")
    return out


def topk_bruteforce(a: np.ndarray, k: int) -> np.ndarray:
    out = np.zeros(k, dtype=np.uint32)
    _check(lib().dgs_oracle_topk_bruteforce(_f32(a), a.size, k, _u32(out)), "topk_bruteforce")
    return out


def worker_step(grad: np.ndarray, state: np.ndarray, offsets: np.ndarray, lr: float, m: float,
                density: float):
    """Updates `state` in place; returns (idx, val)."""
    J = len(offsets) - 1
    _, K = nnz(offsets, density)
    idx = np.zeros(K, dtype=np.uint32)
    val = np.zeros(K, dtype=np.float32)
    out = ctypes.c_uint64(0)
    _check(lib().dgs_oracle_worker_step(_f32(grad), _f32(state), _u64(offsets), J, lr, m,
                                        float(density), _u32(idx), _f32(val), ctypes.byref(out)),
           "worker_step")
    assert out.value == K
    return idx, val


def server_push(model, diff: np.ndarray, idx: np.ndarray, val: np.ndarray) -> None:
    """diff has shape (W, n); model may be None."""
    W, n = diff.shape
    mp = _f32(model) if model is not None else _c_f32p()
    _check(lib().dgs_oracle_server_push(mp, _f32(diff), W, n, _u32(idx), _f32(val), idx.size),
           "server_push")


def server_pull(diff: np.ndarray, k: int, offsets: np.ndarray, density: float):
    """Updates row k of `diff` in place; returns (idx, val)."""
    J = len(offsets) - 1
    _, K = nnz(offsets, density)
    idx = np.zeros(K, dtype=np.uint32)
    val = np.zeros(K, dtype=np.float32)
    out = ctypes.c_uint64(0)
    row = diff[k]
    assert row.flags.c_contiguous
    _check(lib().dgs_oracle_server_pull(_f32(row), _u64(offsets), J, float(density), _u32(idx),
                                        _f32(val), ctypes.byref(out)), "server_pull")
    assert out.value == K
    return idx, val


def server_push_model(model: np.ndarray, idx: np.ndarray, val: np.ndarray) -> None:
    """Printed form of Algorithm 2: the push touches the global model only."""
    _check(lib().dgs_oracle_server_push_model(_f32(model), model.size, _u32(idx), _f32(val), idx.size),
           "server_push_model")


def server_pull_sent(model: np.ndarray, sent: np.ndarray, k: int, offsets: np.ndarray, density: float):
    """Printed form of Algorithm 2: G = top-k of model - sent[k]; sent[k] += G.  Returns (idx, val)."""
    J = len(offsets) - 1
    _, K = nnz(offsets, density)
    idx = np.zeros(K, dtype=np.uint32)
    val = np.zeros(K, dtype=np.float32)
    out = ctypes.c_uint64(0)
    row = sent[k]
    assert row.flags.c_contiguous
    _check(lib().dgs_oracle_server_pull_sent(_f32(model), _f32(row), _u64(offsets), J, float(density),
                                             _u32(idx), _f32(val), ctypes.byref(out)), "server_pull_sent")
    assert out.value == K
    return idx, val


def server_pull_all(diff: np.ndarray, k: int, capacity: int | None = None):
    row = diff[k]
    n = row.size
    cap = n if capacity is None else capacity
    idx = np.zeros(cap, dtype=np.uint32)
    val = np.zeros(cap, dtype=np.float32)
    out = ctypes.c_uint64(0)
    _check(lib().dgs_oracle_server_pull_all(_f32(row), n, _u32(idx), _f32(val), cap,
                                            ctypes.byref(out)), "server_pull_all")
    return idx[:out.value].copy(), val[:out.value].copy()


def server_pull_all_sent(model: np.ndarray, sent: np.ndarray, k: int, capacity: int | None = None):
    row = sent[k]
    n = row.size
    cap = n if capacity is None else capacity
    idx = np.zeros(cap, dtype=np.uint32)
    val = np.zeros(cap, dtype=np.float32)
    out = ctypes.c_uint64(0)
    _check(lib().dgs_oracle_server_pull_all_sent(_f32(model), _f32(row), n, _u32(idx), _f32(val), cap,
                                                 ctypes.byref(out)), "server_pull_all_sent")
    return idx[:out.value].copy(), val[:out.value].copy()


def apply_sparse(dst: np.ndarray, idx: np.ndarray, val: np.ndarray, sign: float = 1.0) -> None:
    _check(lib().dgs_oracle_apply_sparse(_f32(dst), dst.size, _u32(idx), _f32(val), idx.size, sign),
           "apply_sparse")


def wire_bytes(offsets: np.ndarray, density: float) -> int:
    out = ctypes.c_uint64(0)
    _check(lib().dgs_oracle_wire_bytes(_u64(offsets), len(offsets) - 1, float(density), ctypes.byref(out)),
           "wire_bytes")
    return int(out.value)


def encode(offsets: np.ndarray, density: float, idx: np.ndarray, val: np.ndarray) -> np.ndarray:
    """The message's wire form (uint8 array)."""
    _, K = nnz(offsets, density)
    assert idx.size == K and val.size == K
    wire = np.zeros(wire_bytes(offsets, density), dtype=np.uint8)
    _check(lib().dgs_oracle_encode(_u64(offsets), len(offsets) - 1, float(density), _u32(idx), _f32(val),
                                   wire.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))), "encode")
    return wire


def wire_bytes16(offsets: np.ndarray, density: float) -> int:
    out = ctypes.c_uint64(0)
    _check(lib().dgs_oracle_wire_bytes16(_u64(offsets), len(offsets) - 1, float(density), ctypes.byref(out)),
           "wire_bytes16")
    return int(out.value)


def encode16(offsets: np.ndarray, density: float, idx: np.ndarray, val: np.ndarray) -> np.ndarray:
    """The wire form with bfloat16 values (uint8 array)."""
    _, K = nnz(offsets, density)
    assert idx.size == K and val.size == K
    wire = np.zeros(wire_bytes16(offsets, density), dtype=np.uint8)
    _check(lib().dgs_oracle_encode16(_u64(offsets), len(offsets) - 1, float(density), _u32(idx), _f32(val),
                                     wire.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))), "encode16")
    return wire


def decode16(offsets: np.ndarray, density: float, wire: np.ndarray):
    _, K = nnz(offsets, density)
    assert wire.dtype == np.uint8 and wire.flags.c_contiguous and wire.size == wire_bytes16(offsets, density)
    idx = np.zeros(K, dtype=np.uint32)
    val = np.zeros(K, dtype=np.float32)
    _check(lib().dgs_oracle_decode16(_u64(offsets), len(offsets) - 1, float(density),
                                     wire.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), _u32(idx), _f32(val)),
           "decode16")
    return idx, val


def decode(offsets: np.ndarray, density: float, wire: np.ndarray):
    _, K = nnz(offsets, density)
    assert wire.dtype == np.uint8 and wire.flags.c_contiguous and wire.size == wire_bytes(offsets, density)
    idx = np.zeros(K, dtype=np.uint32)
    val = np.zeros(K, dtype=np.float32)
    _check(lib().dgs_oracle_decode(_u64(offsets), len(offsets) - 1, float(density),
                                   wire.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), _u32(idx), _f32(val)),
           "decode")
    return idx, val
