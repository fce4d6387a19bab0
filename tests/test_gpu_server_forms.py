"""GPU parity of the server state as Algorithm 2 prints it (global model plus what each
worker has been sent): dgs_server_push_model / dgs_server_pull_sent against the oracle,
bit-exact indices, values within 1e-6 relative / 1e-7 absolute (the bits agree in fact:
one fp32 subtraction and one fp32 addition on both sides)."""
import numpy as np
import pytest

from paper_1910_10929_amd import dgs, synth
from harness import assert_pairs_match, assert_state_match, to_dev, to_host_u32

pytestmark = pytest.mark.gpu


class SentServer:
    def __init__(self, ctx, model_host, density_max=1.0):
        import torch
        self.ctx = ctx
        dev = ctx.device
        self.model = to_dev(model_host.copy(), dev)
        self.sent = to_dev(np.tile(model_host, (ctx.W, 1)), dev)
        ctx.server_attach_sent(self.sent)
        cap = ctx.nnz(density_max)
        self.idx = torch.zeros(max(cap, 1), dtype=torch.int32, device=dev)
        self.val = torch.zeros(max(cap, 1), dtype=torch.float32, device=dev)

    def push(self, idx_host, val_host):
        di, dv = to_dev(idx_host, self.ctx.device), to_dev(val_host, self.ctx.device)
        self.ctx.server_push_model(self.model, di, dv, idx_host.size)

    def pull(self, worker_id, density):
        import torch
        K = self.ctx.server_pull_sent(self.model, worker_id, density, self.idx, self.val)
        torch.cuda.synchronize()
        return to_host_u32(self.idx[:K]), self.val[:K].cpu().numpy()


def run_events(oracle, off, W, events, rho_up, rho_down, seed, seg_mode=None, extra=()):
    n = int(off[-1])
    J = len(off) - 1
    rng = np.random.default_rng(seed)
    scales = synth.tensor_scales(J, seed + 1)
    kj, _ = oracle.nnz(off, rho_up)
    model0 = synth.gaussian(n, rng)
    ctx = dgs.Context(off, W=W)
    ctx.set_option(dgs.OPT_VALIDATE, 1)
    if seg_mode is not None:
        ctx.set_option(dgs.OPT_SEGMENTED, seg_mode)
    srv = SentServer(ctx, model0)
    model_ref = model0.copy()
    sent_ref = np.tile(model0, (W, 1))
    order = synth.event_schedule(W, events, seed + 2)
    for e, k in enumerate(order):
        k = int(k)
        idx, val = synth.sparse_payload(off, kj, scales, rng)
        oracle.server_push_model(model_ref, idx, val)
        srv.push(idx, val)
        wi, wv = oracle.server_pull_sent(model_ref, sent_ref, k, off, rho_down)
        gi, gv = srv.pull(k, rho_down)
        assert_pairs_match(gi, gv, wi, wv, f"event {e} pull({k})")
    for k, rho in extra:                      # pulls with nothing new in between, dense pulls
        wi, wv = oracle.server_pull_sent(model_ref, sent_ref, k, off, rho)
        gi, gv = srv.pull(k, rho)
        assert np.array_equal(gi, wi), f"extra pull({k}, {rho})"
        assert np.array_equal(gv.view(np.uint32), wv.view(np.uint32)), f"extra pull({k}, {rho})"
    assert_state_match(srv.model.cpu().numpy(), model_ref, "model")
    assert_state_match(srv.sent.cpu().numpy().ravel(), sent_ref.ravel(), "sent")
    st = ctx.stats()
    assert st.internal_errors == 0
    ctx.close()
    return st


def test_printed_form_random_interleaving(oracle):
    off = synth.offsets_from_sizes([120_000, 64, 9408, 40_000, 7, 8193])
    run_events(oracle, off, W=5, events=30, rho_up=0.004, rho_down=0.002, seed=60,
               extra=[(0, 0.002), (0, 0.002), (0, 0.002), (1, 0.5), (2, 1.0), (2, 0.01)])


def test_printed_form_segmented(oracle):
    off = synth.offsets_from_sizes([320_000, 64, 9408, 140_000, 7])
    st = run_events(oracle, off, W=3, events=18, rho_up=0.004, rho_down=0.002, seed=63,
                    seg_mode=dgs.SEG_ALWAYS, extra=[(1, 0.002), (1, 0.002), (1, 0.002)])
    assert st.segmented_tensors > 0


def test_printed_form_full_size_resnet50_shapes(oracle):
    """25,557,032 parameters, 8 workers; pushes shaped like worker messages at density 1e-3."""
    off = synth.layout_resnet50()
    st = run_events(oracle, off, W=8, events=10, rho_up=1e-3, rho_down=1e-3, seed=66)
    assert st.exact_calls <= 8


def test_printed_form_without_secondary_compression(oracle):
    """dgs_server_pull_all_sent: every nonzero of model - sent_k, sent_k += G; a ragged layout
    whose last tile is partial, pulls that find nothing, and the capacity error."""
    import torch
    off = synth.offsets_from_sizes([70_001, 64, 9408, 5])
    n = int(off[-1])
    W = 3
    rng = np.random.default_rng(70)
    scales = synth.tensor_scales(len(off) - 1, 71)
    kj, _ = oracle.nnz(off, 0.004)
    model0 = synth.gaussian(n, rng)
    ctx = dgs.Context(off, W=W)
    srv = SentServer(ctx, model0)
    cap = 4 * int(sum(kj)) + 8
    oi = torch.zeros(cap, dtype=torch.int32, device=ctx.device)
    ov = torch.zeros(cap, dtype=torch.float32, device=ctx.device)
    model_ref = model0.copy()
    sent_ref = np.tile(model0, (W, 1))
    for e, k in enumerate((0, 1, 0, 0, 2, 1, 1)):
        if e != 3:                                   # event 3: a pull with nothing new
            idx, val = synth.sparse_payload(off, kj, scales, rng)
            oracle.server_push_model(model_ref, idx, val)
            srv.push(idx, val)
        wi, wv = oracle.server_pull_all_sent(model_ref, sent_ref, k)
        K = ctx.server_pull_all_sent(srv.model, k, oi, ov, cap)
        torch.cuda.synchronize()
        assert K == wi.size, f"event {e}"
        assert np.array_equal(to_host_u32(oi[:K]), wi), f"event {e}"
        assert np.array_equal(ov[:K].cpu().numpy().view(np.uint32), wv.view(np.uint32)), f"event {e}"
    assert_state_match(srv.sent.cpu().numpy().ravel(), sent_ref.ravel(), "sent")
    idx, val = synth.sparse_payload(off, kj, scales, rng)
    srv.push(idx, val)
    before = srv.sent.clone()
    with pytest.raises(dgs.DgsError) as err:
        ctx.server_pull_all_sent(srv.model, 2, oi, ov, 10)
    assert err.value.code == dgs.DGS_ECAPACITY
    torch.cuda.synchronize()
    assert torch.equal(before, srv.sent)             # nothing was modified
    assert ctx.stats().internal_errors == 0
    ctx.close()


def test_printed_form_argument_errors():
    import torch
    off = synth.offsets_from_sizes([5000, 20])
    ctx = dgs.Context(off, W=2)
    L = dgs.lib()
    h = ctx._h
    n = int(off[-1])
    model = torch.zeros(n, device="cuda:0")
    idx = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    val = torch.zeros(64, device="cuda:0")
    assert L.dgs_server_pull_sent(h, model.data_ptr(), 0, 0.01, idx.data_ptr(), val.data_ptr(), None) == dgs.DGS_EINVAL   # not attached
    sent = torch.zeros((2, n), device="cuda:0")
    ctx.server_attach_sent(sent)
    assert L.dgs_server_pull_sent(h, None, 0, 0.01, idx.data_ptr(), val.data_ptr(), None) == dgs.DGS_EINVAL     # no model
    assert L.dgs_server_pull_sent(h, model.data_ptr(), 2, 0.01, idx.data_ptr(), val.data_ptr(), None) == dgs.DGS_EINVAL   # worker id
    assert L.dgs_server_pull_sent(h, model.data_ptr(), 0, 0.0, idx.data_ptr(), val.data_ptr(), None) == dgs.DGS_EINVAL    # density
    assert L.dgs_server_push_model(h, None, idx.data_ptr(), val.data_ptr(), 1) == dgs.DGS_EINVAL
    ctx.set_option(dgs.OPT_VALIDATE, 1)
    bad = to_dev(np.array([9, 9], np.uint32))
    assert L.dgs_server_push_model(h, model.data_ptr(), bad.data_ptr(), val.data_ptr(), 2) == dgs.DGS_EINVAL
    torch.cuda.synchronize()
    assert not model.any().item()
    ctx.close()


@pytest.mark.parametrize("repair_round", [1, 0], ids=["roles", "no-roles"])
@pytest.mark.parametrize("form", ["sent", "diff"])
def test_pulls_trim_complete_but_overlong_lists(oracle, form, repair_round):
    """Dense pushes whose scale grows between pulls, in both server forms: the threshold hinted by
    the previous pull lets several per cent of a 6M-element tensor (two join groups) and of a
    3M-element one (joined by one workgroup) through.  Every candidate is collected, so the
    selecting workgroups cut the lists down against their own histogram -- also with the
    re-collecting roles switched off, where the only other way out would be the slow
    single-workgroup selection."""
    from harness import Server
    off = synth.offsets_from_sizes([6_000_011, 3_000_000, 64])
    n = int(off[-1])
    rho = 1e-3
    rng = np.random.default_rng(71)
    ctx = dgs.Context(off, W=1)
    ctx.set_option(dgs.OPT_REPAIR_ROUND, repair_round)
    everything = np.arange(n, dtype=np.uint32)
    model_ref = np.zeros(n, np.float32)
    if form == "sent":
        srv = SentServer(ctx, model_ref, density_max=rho)
        sent_ref = np.zeros((1, n), np.float32)
    else:
        srv = Server(ctx, model_ref, density_max=rho)
        diff_ref = np.zeros((1, n), np.float32)
    for e, f in enumerate((1, 1, 3)):
        val = synth.gaussian(n, rng) * np.float32(f)
        if form == "sent":
            oracle.server_push_model(model_ref, everything, val)
            srv.push(everything, val)
            wi, wv = oracle.server_pull_sent(model_ref, sent_ref, 0, off, rho)
        else:
            oracle.server_push(model_ref, diff_ref, everything, val)
            srv.push(0, everything, val)
            wi, wv = oracle.server_pull(diff_ref, 0, off, rho)
        gi, gv = srv.pull(0, rho)
        assert_pairs_match(gi, gv, wi, wv, f"{form} pull {e}")
    if form == "sent":
        assert_state_match(srv.sent.cpu().numpy().ravel(), sent_ref.ravel(), "sent")
    else:
        assert_state_match(srv.diff.cpu().numpy().ravel(), diff_ref.ravel(), "difference row")
    st = ctx.stats()
    assert st.internal_errors == 0 and st.repaired_tensors >= 2
    if repair_round == 0:
        assert st.fallback_tensors == 0
    ctx.close()
