"""Thin ctypes binding of libdgs (see include/dgs.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch is used for device memory and streams.  There is no CPU
fallback: if the shared library is missing, importing `lib()` raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdgs.so")

DGS_OK = 0
DGS_EINVAL, DGS_ENOMEM, DGS_ENOTSUP, DGS_ECAPACITY, DGS_EHIP = -1, -2, -3, -4, -5
OPT_FORCE_EXACT, OPT_PROFILE, OPT_VALIDATE, OPT_MARGIN_PCT, OPT_STREAM_QUADS, OPT_SEGMENTED, OPT_REPAIR_ROUND, OPT_SPIN_LIMIT, OPT_WIRE_VALUE_BITS = 1, 2, 3, 4, 5, 6, 7, 8, 9
SEG_AUTO, SEG_ALWAYS, SEG_NEVER = 0, 1, 2
(PROF_WORKER_STREAM, PROF_WORKER_SELECT, PROF_PULL_STREAM, PROF_PULL_SELECT, PROF_PUSH, PROF_EXACT_EXTRA,
 PROF_WORKER_SEGMENTED, PROF_PULL_SEGMENTED, PROF_ENCODE, PROF_DECODE) = range(10)

EXPORTS = [
    "dgs_workspace_bytes", "dgs_create", "dgs_destroy", "dgs_nnz", "dgs_worker_step",
    "dgs_server_attach", "dgs_server_push", "dgs_server_pull", "dgs_server_pull_all",
    "dgs_apply_sparse", "dgs_set_option", "dgs_get_stats", "dgs_profile_read", "dgs_strerror",
    "dgs_server_attach_sent", "dgs_server_push_model", "dgs_server_pull_sent",
    "dgs_wire_bytes", "dgs_encode", "dgs_decode", "dgs_server_pull_all_sent",
    "dgs_worker_step_static",
]


class DgsError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


class _Stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in (
        "calls_worker", "calls_pull", "calls_push", "exact_calls", "fallback_tensors",
        "fallback_elems", "candidates", "internal_errors", "segmented_tensors", "repaired_tensors")]


_lib = None
_vp = ctypes.c_void_p
_u64p = ctypes.POINTER(ctypes.c_uint64)


def lib():
    """Load libdgs.so.  Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1910_10929_amd.build` "
                "(hipcc, gfx950).  libdgs has no CPU fallback.")
        L = ctypes.CDLL(LIB_PATH)
        L.dgs_workspace_bytes.restype = ctypes.c_size_t
        L.dgs_workspace_bytes.argtypes = [_u64p, ctypes.c_uint32, ctypes.c_uint32]
        L.dgs_create.argtypes = [ctypes.POINTER(_vp), _u64p, ctypes.c_uint32, ctypes.c_uint32, _vp,
                                 ctypes.c_size_t, _vp]
        L.dgs_destroy.argtypes = [_vp]
        L.dgs_nnz.argtypes = [_vp, ctypes.c_double, _u64p]
        L.dgs_worker_step.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_float, ctypes.c_float,
                                      ctypes.c_double, _vp, _vp, _u64p]
        L.dgs_worker_step_static.argtypes = [_u64p, ctypes.c_uint32, _vp, _vp, _vp, ctypes.c_float,
                                             ctypes.c_float, ctypes.c_double, _vp, _vp, _u64p, _vp]
        L.dgs_server_attach.argtypes = [_vp, _vp]
        L.dgs_server_push.argtypes = [_vp, _vp, ctypes.c_uint32, _vp, _vp, ctypes.c_uint64]
        L.dgs_server_pull.argtypes = [_vp, ctypes.c_uint32, ctypes.c_double, _vp, _vp, _u64p]
        L.dgs_server_pull_all.argtypes = [_vp, ctypes.c_uint32, _vp, _vp, ctypes.c_uint64, _u64p]
        L.dgs_server_pull_all_sent.argtypes = [_vp, _vp, ctypes.c_uint32, _vp, _vp, ctypes.c_uint64, _u64p]
        L.dgs_apply_sparse.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_uint64, ctypes.c_float]
        L.dgs_wire_bytes.argtypes = [_vp, ctypes.c_double, _u64p]
        L.dgs_encode.argtypes = [_vp, ctypes.c_double, _vp, _vp, _vp]
        L.dgs_decode.argtypes = [_vp, ctypes.c_double, _vp, _vp, _vp]
        L.dgs_server_attach_sent.argtypes = [_vp, _vp]
        L.dgs_server_push_model.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_uint64]
        L.dgs_server_pull_sent.argtypes = [_vp, _vp, ctypes.c_uint32, ctypes.c_double, _vp, _vp, _u64p]
        L.dgs_set_option.argtypes = [_vp, ctypes.c_int, ctypes.c_int64]
        L.dgs_get_stats.argtypes = [_vp, ctypes.POINTER(_Stats)]
        L.dgs_profile_read.argtypes = [_vp, ctypes.c_int, _u64p, ctypes.POINTER(ctypes.c_double)]
        L.dgs_strerror.restype = ctypes.c_char_p
        L.dgs_strerror.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().dgs_strerror(code).decode()


def _check(rc: int, what: str) -> None:
    if rc != DGS_OK:
        raise DgsError(rc, what)


def _offsets_arg(offsets):
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    return off, off.ctypes.data_as(_u64p)


def workspace_bytes(offsets, W: int) -> int:
    off, p = _offsets_arg(offsets)
    return int(lib().dgs_workspace_bytes(p, len(off) - 1, W))


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def worker_step_static(offsets, grad, state, lr: float, m: float, density: float, idx_out, val_out,
                       residual_mode: bool = False, stream=None) -> int:
    """dgs_worker_step_static: the worker step without a context, on the library's static scratch
    (no device allocation inside the call).  Returns K."""
    import torch
    off, p = _offsets_arg(offsets)
    K = ctypes.c_uint64(0)
    mom, res = (None, state) if residual_mode else (state, None)
    st = stream if stream is not None else torch.cuda.current_stream(grad.device)
    _check(lib().dgs_worker_step_static(p, len(off) - 1, _ptr(grad), _ptr(mom), _ptr(res), lr, m, density,
                                        _ptr(idx_out), _ptr(val_out), ctypes.byref(K), st.cuda_stream),
           "dgs_worker_step_static")
    return int(K.value)


@dataclass
class Stats:
    calls_worker: int
    calls_pull: int
    calls_push: int
    exact_calls: int
    fallback_tensors: int
    fallback_elems: int
    candidates: int
    internal_errors: int
    segmented_tensors: int = 0
    repaired_tensors: int = 0


class Context:
    """Owns a dgs_ctx and the torch tensor backing its workspace."""

    def __init__(self, offsets, W: int = 0, device="cuda:0", stream=None):
        import torch
        self._torch = torch
        self.offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
        self.J = len(self.offsets) - 1
        self.n = int(self.offsets[-1])
        self.W = W
        self.device = torch.device(device)
        nbytes = workspace_bytes(self.offsets, W)
        if nbytes == 0:
            raise DgsError(DGS_EINVAL, "dgs_workspace_bytes")
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            base = self.workspace.data_ptr()
            self._ws_ptr = (base + 255) // 256 * 256
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
            h = _vp()
            _check(lib().dgs_create(ctypes.byref(h), self.offsets.ctypes.data_as(_u64p), self.J, W,
                                    self._ws_ptr, nbytes, self.stream.cuda_stream), "dgs_create")
        self._h = h
        self.diff = None

    def close(self):
        if getattr(self, "_h", None):
            lib().dgs_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- queries / options ----------------------------------------------------
    def nnz(self, density: float) -> int:
        K = ctypes.c_uint64(0)
        _check(lib().dgs_nnz(self._h, density, ctypes.byref(K)), "dgs_nnz")
        return int(K.value)

    def set_option(self, option: int, value: int) -> None:
        _check(lib().dgs_set_option(self._h, option, value), "dgs_set_option")

    def stats(self) -> Stats:
        s = _Stats()
        _check(lib().dgs_get_stats(self._h, ctypes.byref(s)), "dgs_get_stats")
        return Stats(*[int(getattr(s, f[0])) for f in _Stats._fields_])

    def profile_read(self, kind: int):
        cnt = ctypes.c_uint64(0)
        ms = ctypes.c_double(0.0)
        _check(lib().dgs_profile_read(self._h, kind, ctypes.byref(cnt), ctypes.byref(ms)), "dgs_profile_read")
        return int(cnt.value), float(ms.value)

    def _check_capacity(self, density, idx_out, val_out) -> None:
        """The C ABI trusts the caller's output capacity; refuse short buffers here."""
        need = self.nnz(density)
        if idx_out.numel() < need or val_out.numel() < need:
            raise DgsError(DGS_ECAPACITY, f"output buffers hold fewer than K={need} pairs")

    # -- the three calls --------------------------------------------------------
    def worker_step(self, grad, state, lr: float, m: float, density: float, idx_out, val_out,
                    residual_mode: bool = False) -> int:
        K = ctypes.c_uint64(0)
        self._check_capacity(density, idx_out, val_out)
        mom, res = (None, state) if residual_mode else (state, None)
        _check(lib().dgs_worker_step(self._h, _ptr(grad), _ptr(mom), _ptr(res), lr, m, density,
                                     _ptr(idx_out), _ptr(val_out), ctypes.byref(K)), "dgs_worker_step")
        return int(K.value)

    def server_attach(self, diff) -> None:
        _check(lib().dgs_server_attach(self._h, _ptr(diff)), "dgs_server_attach")
        self.diff = diff

    def server_push(self, model, worker_id: int, idx, val, nnz: int) -> None:
        _check(lib().dgs_server_push(self._h, _ptr(model), worker_id, _ptr(idx), _ptr(val), nnz),
               "dgs_server_push")

    def server_pull(self, worker_id: int, density: float, idx_out, val_out) -> int:
        K = ctypes.c_uint64(0)
        self._check_capacity(density, idx_out, val_out)
        _check(lib().dgs_server_pull(self._h, worker_id, density, _ptr(idx_out), _ptr(val_out),
                                     ctypes.byref(K)), "dgs_server_pull")
        return int(K.value)

    # -- the server state as Algorithm 2 prints it: global model + what each worker was sent
    def server_attach_sent(self, sent) -> None:
        _check(lib().dgs_server_attach_sent(self._h, _ptr(sent)), "dgs_server_attach_sent")
        self.sent = sent

    def server_push_model(self, model, idx, val, nnz: int) -> None:
        _check(lib().dgs_server_push_model(self._h, _ptr(model), _ptr(idx), _ptr(val), nnz),
               "dgs_server_push_model")

    def server_pull_sent(self, model, worker_id: int, density: float, idx_out, val_out) -> int:
        K = ctypes.c_uint64(0)
        self._check_capacity(density, idx_out, val_out)
        _check(lib().dgs_server_pull_sent(self._h, _ptr(model), worker_id, density, _ptr(idx_out),
                                          _ptr(val_out), ctypes.byref(K)), "dgs_server_pull_sent")
        return int(K.value)

    def server_pull_all(self, worker_id: int, idx_out, val_out, capacity: int) -> int:
        K = ctypes.c_uint64(0)
        rc = lib().dgs_server_pull_all(self._h, worker_id, _ptr(idx_out), _ptr(val_out), capacity,
                                       ctypes.byref(K))
        if rc == DGS_ECAPACITY:
            raise DgsError(rc, f"dgs_server_pull_all needs capacity {K.value}")
        _check(rc, "dgs_server_pull_all")
        return int(K.value)

    def server_pull_all_sent(self, model, worker_id: int, idx_out, val_out, capacity: int) -> int:
        K = ctypes.c_uint64(0)
        rc = lib().dgs_server_pull_all_sent(self._h, _ptr(model), worker_id, _ptr(idx_out), _ptr(val_out),
                                            capacity, ctypes.byref(K))
        if rc == DGS_ECAPACITY:
            raise DgsError(rc, f"dgs_server_pull_all_sent needs capacity {K.value}")
        _check(rc, "dgs_server_pull_all_sent")
        return int(K.value)

    def apply_sparse(self, dst, idx, val, nnz: int, sign: float = 1.0) -> None:
        _check(lib().dgs_apply_sparse(self._h, _ptr(dst), _ptr(idx), _ptr(val), nnz, sign),
               "dgs_apply_sparse")

    # -- wire form of a message ---------------------------------------------------

    def wire_bytes(self, density: float) -> int:
        out = ctypes.c_uint64(0)
        _check(lib().dgs_wire_bytes(self._h, float(density), ctypes.byref(out)), "dgs_wire_bytes")
        return int(out.value)

    def encode(self, density: float, idx, val, wire) -> None:
        """idx, val: the message of `density` (K entries); wire: uint8 device tensor of wire_bytes(density)."""
        K = self.nnz(density)
        if idx.numel() < K or val.numel() < K or wire.numel() * wire.element_size() < self.wire_bytes(density):
            raise DgsError(DGS_ECAPACITY, "dgs_encode: buffers shorter than the message")
        _check(lib().dgs_encode(self._h, float(density), _ptr(idx), _ptr(val), _ptr(wire)), "dgs_encode")

    def decode(self, density: float, wire, idx_out, val_out) -> None:
        K = self.nnz(density)
        if (idx_out.numel() < K or val_out.numel() < K
                or wire.numel() * wire.element_size() < self.wire_bytes(density)):
            raise DgsError(DGS_ECAPACITY, "dgs_decode: buffers shorter than the message")
        _check(lib().dgs_decode(self._h, float(density), _ptr(wire), _ptr(idx_out), _ptr(val_out)), "dgs_decode")
