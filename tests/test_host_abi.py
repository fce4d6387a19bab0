"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and the pure-host entry points behave."""
import ctypes
import os
import re

import numpy as np

from paper_1910_10929_amd import dgs as libdgs, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dgs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dgs_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared_symbols()
    assert "dgs_worker_step" in names and "dgs_server_push" in names and "dgs_server_pull" in names
    L = libdgs.lib()
    for name in names:
        assert hasattr(L, name), f"libdgs.so does not export {name}"
    assert sorted(libdgs.EXPORTS) == names


def test_strerror_and_workspace_bytes():
    assert libdgs.strerror(0) == "ok"
    assert "invalid" in libdgs.strerror(-1)
    off = synth.layout_resnet50()
    nbytes = libdgs.workspace_bytes(off, 32)
    n = int(off[-1])
    assert 4 * n < nbytes < 6 * n          # about 4 B per parameter of scratch
    # invalid layouts give 0
    assert libdgs.workspace_bytes(np.array([0, 5, 5], np.uint64), 0) == 0      # empty tensor
    assert libdgs.workspace_bytes(np.array([1, 5], np.uint64), 0) == 0         # does not start at 0
    assert libdgs.workspace_bytes(np.array([0, 1 << 32], np.uint64), 0) == 0   # index width
    L = libdgs.lib()
    assert L.dgs_workspace_bytes(None, 3, 0) == 0


def test_null_context_is_rejected():
    L = libdgs.lib()
    K = ctypes.c_uint64(0)
    assert L.dgs_nnz(None, 0.5, ctypes.byref(K)) == libdgs.DGS_EINVAL
    assert L.dgs_destroy(None) == libdgs.DGS_EINVAL
    assert L.dgs_set_option(None, 1, 1) == libdgs.DGS_EINVAL
    h = ctypes.c_void_p()
    off = np.array([0, 8], np.uint64)
    rc = L.dgs_create(ctypes.byref(h), off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), 1, 0,
                      None, 0, None)
    assert rc == libdgs.DGS_EINVAL and not h.value
