"""GPU parity on seeded random layouts: tensor sizes from 1 to 400k in random order,
random densities, momentum and learning rates, worker steps followed by pushes and
pulls through both server forms, on the default code-path choice and with the
multi-workgroup selection forced.  Every case is compared with the oracle element by
element (indices bit-exact, values 1e-6 relative / 1e-7 absolute, state bits equal)."""
import numpy as np
import pytest

from paper_1910_10929_amd import dgs, synth
from harness import Server, Worker, assert_pairs_match, assert_state_match, to_dev, to_host_u32

pytestmark = pytest.mark.gpu


def random_layout(rng):
    J = int(rng.integers(1, 12))
    kinds = rng.integers(0, 4, size=J)
    sizes = []
    for kd in kinds:
        if kd == 0:
            sizes.append(int(rng.integers(1, 300)))
        elif kd == 1:
            sizes.append(int(rng.integers(300, 9000)))
        elif kd == 2:
            sizes.append(int(rng.integers(9000, 70_000)))
        else:
            sizes.append(int(rng.integers(70_000, 400_000)))
    return sizes


@pytest.mark.parametrize("seed", list(range(30)))
def test_random_layout_worker_and_server(oracle, seed):
    import torch
    rng = np.random.default_rng(1000 + seed)
    sizes = random_layout(rng)
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    J = len(sizes)
    rho_up = float(rng.choice([1e-3, 3e-3, 0.01, 0.03, 0.2]))
    rho_down = float(rng.choice([1e-3, 5e-3, 0.02]))
    m = np.float32(rng.choice([0.0, 0.5, 0.9]))
    lr = np.float32(rng.choice([1.0, 0.1]))
    scales = synth.tensor_scales(J, 2000 + seed)
    heavy = bool(rng.integers(0, 2))
    seg_mode = [None, dgs.SEG_ALWAYS, dgs.SEG_NEVER][seed % 3]
    W = 2
    ctx = dgs.Context(off, W=W)
    if seg_mode is not None:
        ctx.set_option(dgs.OPT_SEGMENTED, seg_mode)
    w = Worker(ctx, density_max=max(rho_up, rho_down))
    srv = Server(ctx, np.zeros(n, np.float32), density_max=max(rho_up, rho_down))
    sent_dev = torch.zeros((W, n), dtype=torch.float32, device="cuda:0")
    model2_dev = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    s_ref = np.zeros(n, np.float32)
    model_ref = np.zeros(n, np.float32)
    diff_ref = np.zeros((W, n), np.float32)
    model2_ref = np.zeros(n, np.float32)
    sent_ref = np.zeros((W, n), np.float32)
    # second context for the printed server form (the two forms share hint sets per worker id)
    ctx2 = dgs.Context(off, W=W)
    if seg_mode is not None:
        ctx2.set_option(dgs.OPT_SEGMENTED, seg_mode)
    ctx2.server_attach_sent(sent_dev)
    pidx = torch.zeros(max(ctx.nnz(max(rho_up, rho_down)), 1), dtype=torch.int32, device="cuda:0")
    pval = torch.zeros(pidx.numel(), dtype=torch.float32, device="cuda:0")
    for t in range(4):
        g = synth.student_t_grads(off, scales, rng) if heavy else synth.gaussian_grads(off, scales, rng)
        if t == 2:
            g[: n // 3] = 0.0                      # a block of exact zeros
        wi, wv = oracle.worker_step(g, s_ref, off, lr, m, rho_up)
        gi, gv = w.step(g, lr, m, rho_up, residual_mode=(m == 0.0 and seed % 2 == 0))
        assert_pairs_match(gi, gv, wi, wv, f"seed {seed} step {t} sizes {sizes}")
        assert_state_match(w.state_host(), s_ref, f"seed {seed} state {t}")
        k = t % W
        oracle.server_push(model_ref, diff_ref, wi, wv)
        ctx.server_push(srv.model, k, w.idx, w.val, gi.size)
        pi_ref, pv_ref = oracle.server_pull(diff_ref, k, off, rho_down)
        pi, pv = srv.pull(k, rho_down)
        assert_pairs_match(pi, pv, pi_ref, pv_ref, f"seed {seed} pull {t}")
        oracle.server_push_model(model2_ref, wi, wv)
        ctx2.server_push_model(model2_dev, w.idx, w.val, gi.size)
        qi_ref, qv_ref = oracle.server_pull_sent(model2_ref, sent_ref, k, off, rho_down)
        K = ctx2.server_pull_sent(model2_dev, k, rho_down, pidx, pval)
        torch.cuda.synchronize()
        assert_pairs_match(to_host_u32(pidx[:K]), pval[:K].cpu().numpy(), qi_ref, qv_ref,
                           f"seed {seed} pull_sent {t}")
    assert_state_match(srv.model.cpu().numpy(), model_ref, "model")
    assert_state_match(srv.diff.cpu().numpy().ravel(), diff_ref.ravel(), "diff")
    assert_state_match(model2_dev.cpu().numpy(), model2_ref, "model (printed form)")
    assert_state_match(sent_dev.cpu().numpy().ravel(), sent_ref.ravel(), "sent")
    assert ctx.stats().internal_errors == 0 and ctx2.stats().internal_errors == 0
    ctx.close()
    ctx2.close()
