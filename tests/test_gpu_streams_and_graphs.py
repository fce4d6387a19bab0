"""Launch modes around the same calls.  (1) One whole step (dgs_worker_step + dgs_server_push +
dgs_server_pull) captured into a HIP graph on the context's stream and replayed: every replay
must give what the oracle gives for that step, with eager work and synchronisations between the
replays; the calls enqueue kernels only (no memset or copy nodes, no host wait) once the plan of a
density is cached.  (2) Worker and server as two contexts on two streams, overlapping."""
import numpy as np
import pytest

from paper_1910_10929_amd import dgs, synth
from harness import assert_pairs_match, assert_state_match, to_host_u32

pytestmark = pytest.mark.gpu


def test_step_replayed_from_a_graph(oracle):
    import torch
    sizes = [300_000, 64, 9408, 70_001, 5]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    rho = 0.004
    lr, m = np.float32(0.5), np.float32(0.9)
    scales = synth.tensor_scales(len(sizes), 80)
    rng = np.random.default_rng(81)
    dev = "cuda:0"
    s = torch.cuda.Stream(device=dev)
    ctx = dgs.Context(off, W=1, device=dev, stream=s)
    K = ctx.nnz(rho)
    with torch.cuda.stream(s):
        g_static = torch.zeros(n, device=dev)
        state = torch.zeros(n, device=dev)
        model = torch.zeros(n, device=dev)
        diff = torch.zeros((1, n), device=dev)
        idx = torch.zeros(K, dtype=torch.int32, device=dev)
        val = torch.zeros(K, device=dev)
        pidx = torch.zeros(K, dtype=torch.int32, device=dev)
        pval = torch.zeros(K, device=dev)
    ctx.server_attach(diff)
    s_ref = np.zeros(n, np.float32)
    model_ref = np.zeros(n, np.float32)
    diff_ref = np.zeros((1, n), np.float32)

    def enqueue():
        ctx.worker_step(g_static, state, float(lr), float(m), rho, idx, val)
        ctx.server_push(model, 0, idx, val, K)
        ctx.server_pull(0, rho, pidx, pval)

    def check(tag, g):
        wi, wv = oracle.worker_step(g, s_ref, off, lr, m, rho)
        oracle.server_push(model_ref, diff_ref, wi, wv)
        pi, pv = oracle.server_pull(diff_ref, 0, off, rho)
        s.synchronize()
        assert_pairs_match(to_host_u32(idx), val.cpu().numpy(), wi, wv, f"{tag}: worker message")
        assert_pairs_match(to_host_u32(pidx), pval.cpu().numpy(), pi, pv, f"{tag}: pull message")
        assert_state_match(state.cpu().numpy(), s_ref, f"{tag}: worker state")
        assert_state_match(diff[0].cpu().numpy(), diff_ref[0], f"{tag}: difference row")

    grads = [synth.gaussian_grads(off, scales, rng) for _ in range(8)]
    with torch.cuda.stream(s):
        for t in range(2):                       # eager: the non-predicted first call, then a predicted one
            g_static.copy_(torch.from_numpy(grads[t]))
            enqueue()
            check(f"eager {t}", grads[t])
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            enqueue()
        for t in range(2, 8):
            g_static.copy_(torch.from_numpy(grads[t]))
            graph.replay()
            check(f"replay {t}", grads[t])
            (state.abs().sum() + model.sum()).item()          # eager work and a host wait in between
    assert_state_match(model.cpu().numpy(), model_ref, "model")
    st = ctx.stats()
    assert st.internal_errors == 0 and st.exact_calls == 2
    ctx.close()


def test_an_unplanned_density_is_refused_during_capture(oracle):
    """Planning a density copies its tables to the device, which a stream capture must not contain:
    a call with a density that has no cached plan returns DGS_ENOTSUP while the stream is being
    captured, and nothing of it is recorded.  The plan that WAS used during a capture survives any
    number of other densities afterwards: the replay keeps giving the oracle's result."""
    import torch
    sizes = [200_000, 64, 9408]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    rho = 0.004
    lr, m = np.float32(1.0), np.float32(0.0)
    dev = "cuda:0"
    s = torch.cuda.Stream(device=dev)
    ctx = dgs.Context(off, W=0, device=dev, stream=s)
    K = ctx.nnz(rho)
    rng = np.random.default_rng(82)
    grads = [synth.gaussian(n, rng) for _ in range(4)]
    with torch.cuda.stream(s):
        g_static = torch.zeros(n, device=dev)
        state = torch.zeros(n, device=dev)
        idx = torch.zeros(2 * K, dtype=torch.int32, device=dev)
        val = torch.zeros(2 * K, device=dev)
        s_ref = np.zeros(n, np.float32)
        for t in range(2):
            g_static.copy_(torch.from_numpy(grads[t]))
            ctx.worker_step(g_static, state, float(lr), float(m), rho, idx, val, residual_mode=True)
            oracle.worker_step(grads[t], s_ref, off, lr, m, rho)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            with pytest.raises(dgs.DgsError) as e:
                ctx.worker_step(g_static, state, float(lr), float(m), 0.0071, idx, val, residual_mode=True)
            assert e.value.code == dgs.DGS_ENOTSUP
            ctx.worker_step(g_static, state, float(lr), float(m), rho, idx, val, residual_mode=True)
        # nine other densities, eagerly: more than the cache holds
        scratch = torch.zeros(n, device=dev)
        for i in range(9):
            ctx.worker_step(g_static, scratch, float(lr), float(m), 0.001 + 0.0005 * i, idx, val, residual_mode=True)
        for t in range(2, 4):
            g_static.copy_(torch.from_numpy(grads[t]))
            graph.replay()
            wi, wv = oracle.worker_step(grads[t], s_ref, off, lr, m, rho)
            s.synchronize()
            assert_pairs_match(to_host_u32(idx)[:K], val.cpu().numpy()[:K], wi, wv, f"replay {t}")
            assert_state_match(state.cpu().numpy(), s_ref, f"replay {t}: state")
    assert ctx.stats().internal_errors == 0
    ctx.close()


def test_worker_and_server_on_two_streams(oracle):
    """Two contexts on two streams of default priority: the worker's step t+1 is enqueued while
    the server still handles push / pull t; messages are double-buffered and ordered with
    events.  Everything is compared at the end, after a single wait."""
    import torch
    sizes = [300_000, 64, 9408, 70_001, 5]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    rho = 0.004
    lr, m = np.float32(0.5), np.float32(0.9)
    scales = synth.tensor_scales(len(sizes), 82)
    rng = np.random.default_rng(83)
    dev = "cuda:0"
    sa, sb = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
    wctx = dgs.Context(off, W=0, device=dev, stream=sa)
    sctx = dgs.Context(off, W=1, device=dev, stream=sb)
    K = wctx.nnz(rho)
    steps = 8
    grads = [synth.gaussian_grads(off, scales, rng) for _ in range(steps)]
    g_dev = [torch.from_numpy(g).to(dev) for g in grads]
    state = torch.zeros(n, device=dev)
    model = torch.zeros(n, device=dev)
    diff = torch.zeros((1, n), device=dev)
    sctx.server_attach(diff)
    msg = [(torch.zeros(K, dtype=torch.int32, device=dev), torch.zeros(K, device=dev)) for _ in range(2)]
    pidx = torch.zeros(K, dtype=torch.int32, device=dev)
    pval = torch.zeros(K, device=dev)
    sent_log = [(torch.zeros(K, dtype=torch.int32, device=dev), torch.zeros(K, device=dev)) for _ in range(steps)]
    pull_log = [(torch.zeros(K, dtype=torch.int32, device=dev), torch.zeros(K, device=dev)) for _ in range(steps)]
    produced = [torch.cuda.Event() for _ in range(2)]
    consumed = [torch.cuda.Event() for _ in range(2)]
    torch.cuda.synchronize()
    for t in range(steps):
        b = t % 2
        if t >= 2:
            sa.wait_event(consumed[b])
        wctx.worker_step(g_dev[t], state, float(lr), float(m), rho, msg[b][0], msg[b][1])
        produced[b].record(sa)
        sb.wait_event(produced[b])
        with torch.cuda.stream(sb):
            sent_log[t][0].copy_(msg[b][0])
            sent_log[t][1].copy_(msg[b][1])
        sctx.server_push(model, 0, msg[b][0], msg[b][1], K)
        consumed[b].record(sb)
        sctx.server_pull(0, rho, pidx, pval)
        with torch.cuda.stream(sb):
            pull_log[t][0].copy_(pidx)
            pull_log[t][1].copy_(pval)
    torch.cuda.synchronize()
    s_ref = np.zeros(n, np.float32)
    model_ref = np.zeros(n, np.float32)
    diff_ref = np.zeros((1, n), np.float32)
    for t in range(steps):
        wi, wv = oracle.worker_step(grads[t], s_ref, off, lr, m, rho)
        oracle.server_push(model_ref, diff_ref, wi, wv)
        pi, pv = oracle.server_pull(diff_ref, 0, off, rho)
        assert_pairs_match(to_host_u32(sent_log[t][0]), sent_log[t][1].cpu().numpy(), wi, wv, f"step {t}: worker message")
        assert_pairs_match(to_host_u32(pull_log[t][0]), pull_log[t][1].cpu().numpy(), pi, pv, f"step {t}: pull message")
    assert_state_match(state.cpu().numpy(), s_ref, "worker state")
    assert_state_match(model.cpu().numpy(), model_ref, "model")
    assert_state_match(diff[0].cpu().numpy(), diff_ref[0], "difference row")
    assert wctx.stats().internal_errors == 0 and sctx.stats().internal_errors == 0
    wctx.close()
    sctx.close()
