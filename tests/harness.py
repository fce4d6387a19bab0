"""Helpers for the GPU parity tests: numpy <-> device plumbing around the
C-ABI binding.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np


def to_dev(a: np.ndarray, device="cuda:0"):
    import torch
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(device)
    return torch.from_numpy(a).to(device)


def to_host_u32(t) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32)


class Worker:
    """One worker's device-resident state + output buffers."""

    def __init__(self, ctx, density_max: float = 1.0, misalign: int = 0):
        import torch
        self.ctx = ctx
        n = ctx.n
        cap = ctx.nnz(density_max)
        dev = ctx.device
        self._state_store = torch.zeros(n + 8, dtype=torch.float32, device=dev)
        self.state = self._state_store[misalign:misalign + n]
        self._grad_store = torch.zeros(n + 8, dtype=torch.float32, device=dev)
        self.grad = self._grad_store[misalign:misalign + n]
        self.idx = torch.zeros(max(cap, 1), dtype=torch.int32, device=dev)
        self.val = torch.zeros(max(cap, 1), dtype=torch.float32, device=dev)

    def step(self, grad_host: np.ndarray, lr, m, density, residual_mode=False):
        import torch
        self.grad.copy_(torch.from_numpy(grad_host))
        K = self.ctx.worker_step(self.grad, self.state, lr, m, density, self.idx, self.val,
                                 residual_mode=residual_mode)
        torch.cuda.synchronize()
        return to_host_u32(self.idx[:K]), self.val[:K].cpu().numpy()

    def state_host(self) -> np.ndarray:
        return self.state.cpu().numpy()


class Server:
    def __init__(self, ctx, model_host: np.ndarray | None, density_max: float = 1.0):
        import torch
        self.ctx = ctx
        dev = ctx.device
        self.diff = torch.zeros((ctx.W, ctx.n), dtype=torch.float32, device=dev)
        ctx.server_attach(self.diff)
        self.model = to_dev(model_host, dev) if model_host is not None else None
        cap = ctx.nnz(density_max)
        self.idx = torch.zeros(max(cap, 1), dtype=torch.int32, device=dev)
        self.val = torch.zeros(max(cap, 1), dtype=torch.float32, device=dev)

    def push(self, worker_id: int, idx_host: np.ndarray, val_host: np.ndarray):
        di, dv = to_dev(idx_host, self.ctx.device), to_dev(val_host, self.ctx.device)
        self.ctx.server_push(self.model, worker_id, di, dv, idx_host.size)
        return di, dv

    def pull(self, worker_id: int, density: float):
        import torch
        K = self.ctx.server_pull(worker_id, density, self.idx, self.val)
        torch.cuda.synchronize()
        return to_host_u32(self.idx[:K]), self.val[:K].cpu().numpy()

    def pull_all(self, worker_id: int, capacity: int | None = None):
        import torch
        cap = self.idx.numel() if capacity is None else capacity
        K = self.ctx.server_pull_all(worker_id, self.idx, self.val, cap)
        torch.cuda.synchronize()
        return to_host_u32(self.idx[:K]), self.val[:K].cpu().numpy()


def assert_pairs_match(idx, val, want_idx, want_val, what=""):
    """Parity bar: indices and nnz bit-exact; fp32 values within 1e-6 relative /
    1e-7 absolute."""
    assert idx.size == want_idx.size, f"{what}: nnz {idx.size} != {want_idx.size}"
    if not np.array_equal(idx, want_idx):
        bad = np.nonzero(idx != want_idx)[0]
        raise AssertionError(f"{what}: {bad.size} index mismatches, first at {bad[0]}: "
                             f"{idx[bad[0]]} != {want_idx[bad[0]]}")
    np.testing.assert_allclose(val, want_val, rtol=1e-6, atol=1e-7, err_msg=what)


def assert_state_match(got: np.ndarray, want: np.ndarray, what=""):
    np.testing.assert_allclose(got, want, rtol=1e-6, atol=1e-7, err_msg=what)
    # the arithmetic is the same single-rounding fma / multiply on both sides,
    # so the bits agree as well
    if not np.array_equal(bits(got), bits(want)):
        bad = np.nonzero(bits(got) != bits(want))[0]
        raise AssertionError(f"{what}: {bad.size} state words differ in bits, first at {bad[0]}")


def run_worker_parity(oracle, off, grads, lr, m, rho, *, force_exact=False, residual=False,
                      misalign=0, margin=None, init_state=None, seg_mode=None, repair_round=None):
    """Several steps of dgs_worker_step vs the oracle; returns the GPU context stats."""
    from paper_1910_10929_amd import dgs
    ctx = dgs.Context(off, W=0)
    if force_exact:
        ctx.set_option(dgs.OPT_FORCE_EXACT, int(force_exact))      # True: two passes; 2: sampled estimate
    if margin is not None:
        ctx.set_option(dgs.OPT_MARGIN_PCT, margin)
    if seg_mode is not None:
        ctx.set_option(dgs.OPT_SEGMENTED, seg_mode)
    if repair_round is not None:
        ctx.set_option(dgs.OPT_REPAIR_ROUND, repair_round)
    w = Worker(ctx, density_max=rho, misalign=misalign)
    n = int(off[-1])
    s_ref = np.zeros(n, np.float32) if init_state is None else init_state.copy()
    if init_state is not None:
        import torch
        w.state.copy_(torch.from_numpy(init_state))
    for t, g in enumerate(grads):
        want_i, want_v = oracle.worker_step(g, s_ref, off, lr, m, rho)
        got_i, got_v = w.step(g, lr, m, rho, residual_mode=residual)
        assert_pairs_match(got_i, got_v, want_i, want_v, f"step {t}")
        assert_state_match(w.state_host(), s_ref, f"state after step {t}")
    st = ctx.stats()
    assert st.internal_errors == 0
    ctx.close()
    return st
