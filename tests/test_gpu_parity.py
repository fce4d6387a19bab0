"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on identical seeded inputs.  Bar: indices and nnz bit-exact; fp32 values within
1e-6 relative / 1e-7 absolute (in fact the bits agree, and the state check
asserts that too)."""
import numpy as np
import pytest

from paper_1910_10929_amd import dgs, synth
from harness import (Server, Worker, assert_pairs_match, assert_state_match, run_worker_parity, to_dev,
                     to_host_u32)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    dgs.lib()   # fails loudly if libdgs.so is missing
    return torch


RAGGED_SIZES = [1, 7, 64, 1000, 8192, 8193, 9408, 3, 100_003, 50_000, 1 << 18, 17, 65_537, 12_345]


def test_c1_flat_one_million(oracle, torch_mod):
    """Config 1: n = 2^20, one tensor, N(0,1), m = 0.9, lr = 1, density 0.01,
    ten rounds of step -> push -> pull -> apply with one worker."""
    torch = torch_mod
    n = 1 << 20
    off = synth.layout_flat(n)
    rng = np.random.default_rng(0)
    ctx = dgs.Context(off, W=1)
    w = Worker(ctx, density_max=0.01)
    srv = Server(ctx, np.zeros(n, np.float32), density_max=0.01)
    theta = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    s_ref = np.zeros(n, np.float32)
    model_ref = np.zeros(n, np.float32)
    diff_ref = np.zeros((1, n), np.float32)
    theta_ref = np.zeros(n, np.float32)
    for t in range(10):
        g = synth.gaussian(n, rng)
        wi, wv = oracle.worker_step(g, s_ref, off, 1.0, np.float32(0.9), 0.01)
        gi, gv = w.step(g, 1.0, 0.9, 0.01)
        assert gi.size == 10486
        assert_pairs_match(gi, gv, wi, wv, f"worker step {t}")
        assert_state_match(w.state_host(), s_ref, f"worker state {t}")
        oracle.server_push(model_ref, diff_ref, wi, wv)
        ctx.server_push(srv.model, 0, w.idx, w.val, gi.size)
        pi_ref, pv_ref = oracle.server_pull(diff_ref, 0, off, 0.01)
        pi, pv = srv.pull(0, 0.01)
        assert_pairs_match(pi, pv, pi_ref, pv_ref, f"pull {t}")
        oracle.apply_sparse(theta_ref, pi_ref, pv_ref, 1.0)
        ctx.apply_sparse(theta, srv.idx, srv.val, pi.size, 1.0)
        torch.cuda.synchronize()
        assert_state_match(srv.model.cpu().numpy(), model_ref, f"model {t}")
        assert_state_match(srv.diff.cpu().numpy()[0], diff_ref[0], f"diff {t}")
        assert_state_match(theta.cpu().numpy(), theta_ref, f"theta {t}")
    st = ctx.stats()
    assert st.internal_errors == 0
    ctx.close()


@pytest.mark.parametrize("force_exact", [False, True, 2], ids=["predicted", "exact", "sampled"])
@pytest.mark.parametrize("rho", [0.001, 0.01, 0.03])
def test_ragged_multi_tensor(oracle, torch_mod, rho, force_exact):
    """Unaligned tensor borders, tiny and large tensors, a ragged tail tile."""
    off = synth.offsets_from_sizes(RAGGED_SIZES)
    scales = synth.tensor_scales(len(RAGGED_SIZES), 21)
    rng = np.random.default_rng(22)
    grads = [synth.gaussian_grads(off, scales, rng) for _ in range(6)]
    st = run_worker_parity(oracle, off, grads, np.float32(0.5), np.float32(0.9), rho,
                           force_exact=force_exact)
    if force_exact:
        assert st.exact_calls == 6
    else:
        assert st.exact_calls == 1     # only the first step has no prediction


def test_predicted_and_exact_paths_agree_bytewise(oracle, torch_mod):
    """Determinism across code paths and across repeated runs."""
    off = synth.offsets_from_sizes([300_000, 64, 70_001])
    rng = np.random.default_rng(23)
    grads = [synth.gaussian(int(off[-1]), rng) for _ in range(5)]
    outs = []
    for force in (0, 1, 0, 2):          # predicted, two passes, predicted again, sampled estimate on every call
        ctx = dgs.Context(off, W=0)
        ctx.set_option(dgs.OPT_FORCE_EXACT, force)
        w = Worker(ctx, density_max=0.005)
        run = []
        for g in grads:
            i, v = w.step(g, 0.1, 0.7, 0.005)
            run.append((i.copy(), v.copy(), w.state_host()))
        outs.append(run)
        ctx.close()
    for a, b in ((outs[0], outs[1]), (outs[0], outs[2]), (outs[0], outs[3])):
        for (i1, v1, s1), (i2, v2, s2) in zip(a, b):
            assert np.array_equal(i1, i2)
            assert np.array_equal(v1.view(np.uint32), v2.view(np.uint32))
            assert np.array_equal(s1.view(np.uint32), s2.view(np.uint32))


def test_misaligned_buffers_take_the_scalar_path(oracle, torch_mod):
    off = synth.offsets_from_sizes([20_000, 5, 40_001])
    rng = np.random.default_rng(24)
    grads = [synth.gaussian(int(off[-1]), rng) for _ in range(3)]
    run_worker_parity(oracle, off, grads, 1.0, np.float32(0.9), 0.01, misalign=1)


def _tie_inputs(n_big):
    rng = np.random.default_rng(25)
    cases = {}
    cases["all_equal"] = np.full(n_big, 1.5, np.float32)
    cases["all_zero"] = np.zeros(n_big, np.float32)
    few = np.zeros(n_big, np.float32)
    few[rng.choice(n_big, 40, replace=False)] = rng.standard_normal(40).astype(np.float32)
    cases["fewer_nonzeros_than_k"] = few
    lv = rng.integers(-3, 4, size=n_big).astype(np.float32)
    cases["few_levels"] = lv
    pm = rng.standard_normal(n_big // 2).astype(np.float32)
    cases["plus_minus_pairs"] = np.concatenate([pm, -pm, np.zeros(n_big - 2 * (n_big // 2), np.float32)])
    sub = (rng.integers(-1000, 1000, size=n_big).astype(np.float32) * np.float32(1e-45))
    cases["subnormals"] = sub
    sp = rng.standard_normal(n_big).astype(np.float32)
    sp[::7] = np.inf
    sp[3::1001] = np.nan
    cases["inf_nan"] = sp
    return cases


@pytest.mark.parametrize("name", ["all_equal", "all_zero", "fewer_nonzeros_than_k", "few_levels",
                                  "plus_minus_pairs", "subnormals", "inf_nan"])
def test_degenerate_value_patterns(oracle, torch_mod, name):
    """Giant tie classes, zeros, subnormals and specials, in a big tensor
    (candidate path + dense re-selection) next to a small one."""
    n_big = 70_000
    g_big = _tie_inputs(n_big)[name]
    off = synth.offsets_from_sizes([n_big, 100, 9000])
    rng = np.random.default_rng(26)
    tail = synth.gaussian(9100, rng)
    g1 = np.concatenate([g_big, tail])
    g2 = np.concatenate([g_big[::-1].copy(), -tail])
    if name == "inf_nan":
        # compare through bits: NaN payloads must match too
        ctx = dgs.Context(off, W=0)
        w = Worker(ctx, density_max=0.002)
        s_ref = np.zeros(int(off[-1]), np.float32)
        wi, wv = oracle.worker_step(g1, s_ref, off, 1.0, np.float32(0.5), 0.002)
        gi, gv = w.step(g1, 1.0, 0.5, 0.002)
        assert np.array_equal(gi, wi)
        assert np.array_equal(gv.view(np.uint32), wv.view(np.uint32))
        assert np.array_equal(w.state_host().view(np.uint32), s_ref.view(np.uint32))
        assert ctx.stats().internal_errors == 0
        ctx.close()
        return
    run_worker_parity(oracle, off, [g1, g2, g1], 1.0, np.float32(0.5), 0.002)
    run_worker_parity(oracle, off, [g1, g2], 1.0, np.float32(0.5), 0.002, force_exact=True)


@pytest.mark.parametrize("rho", [1.0, 0.5, 0.05])
def test_dense_requests(oracle, torch_mod, rho):
    off = synth.offsets_from_sizes([30_000, 1, 999, 20_480])
    rng = np.random.default_rng(27)
    grads = [synth.gaussian(int(off[-1]), rng) for _ in range(3)]
    run_worker_parity(oracle, off, grads, np.float32(0.3), np.float32(0.9), rho)


def test_residual_mode_is_algorithm_1(oracle, torch_mod):
    off = synth.offsets_from_sizes([50_000, 333])
    rng = np.random.default_rng(28)
    grads = [synth.gaussian(int(off[-1]), rng) for _ in range(4)]
    run_worker_parity(oracle, off, grads, np.float32(0.05), 0.0, 0.01, residual=True)


def test_threshold_drop_forces_reselection(oracle, torch_mod):
    """A gradient scale that collapses makes the predicted threshold useless:
    the result must still be exact (dense re-selection), and the next steps
    recover the fast path."""
    off = synth.offsets_from_sizes([200_000, 64])
    n = int(off[-1])
    rng = np.random.default_rng(29)
    g = [synth.gaussian(n, rng) for _ in range(6)]
    state0 = (synth.gaussian(n, rng) * np.float32(1e-3)).astype(np.float32)
    # momentum 0 -> state is the residual; scale the gradients down sharply at step 2
    grads = [g[0], g[1], g[2] * np.float32(1e-6), g[3] * np.float32(1e-6), g[4], g[5]]
    st = run_worker_parity(oracle, off, grads, 1.0, np.float32(0.0), 0.001, residual=True,
                           init_state=state0)
    assert st.internal_errors == 0


def test_server_many_workers_random_interleaving(oracle, torch_mod):
    """W = 6 asynchronous workers simulated as a seeded sequence of push + pull
    events against one GPU-resident server state."""
    torch = torch_mod
    sizes = [120_000, 64, 9408, 40_000, 7]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    W = 6
    rho_up, rho_down = 0.004, 0.002
    scales = synth.tensor_scales(len(sizes), 31)
    rng = np.random.default_rng(32)
    kj, K = oracle.nnz(off, rho_up)
    ctx = dgs.Context(off, W=W)
    ctx.set_option(dgs.OPT_VALIDATE, 1)
    model0 = synth.gaussian(n, rng)
    srv = Server(ctx, model0.copy(), density_max=1.0)
    model_ref = model0.copy()
    diff_ref = np.zeros((W, n), np.float32)
    order = synth.event_schedule(W, 30, 33)
    for e, k in enumerate(order):
        k = int(k)
        idx, val = synth.sparse_payload(off, kj, scales, rng)
        oracle.server_push(model_ref, diff_ref, idx, val)
        srv.push(k, idx, val)
        wi, wv = oracle.server_pull(diff_ref, k, off, rho_down)
        gi, gv = srv.pull(k, rho_down)
        assert_pairs_match(gi, gv, wi, wv, f"event {e} pull({k})")
    torch.cuda.synchronize()
    assert_state_match(srv.model.cpu().numpy(), model_ref, "model")
    assert_state_match(srv.diff.cpu().numpy().ravel(), diff_ref.ravel(), "diff")
    # pull before anything was pushed to a fresh row / fewer than k nonzeros
    wi, wv = oracle.server_pull(diff_ref, 0, off, 0.5)
    gi, gv = srv.pull(0, 0.5)
    assert_pairs_match(gi, gv, wi, wv, "dense pull")
    # without secondary compression: everything that is left
    wi, wv = oracle.server_pull_all(diff_ref, 1)
    gi, gv = srv.pull_all(1, capacity=n)
    assert_pairs_match(gi, gv, wi, wv, "pull_all")
    assert not srv.diff[1].any().item()
    assert ctx.stats().internal_errors == 0
    ctx.close()


def test_pull_on_empty_difference_and_capacity_error(oracle, torch_mod):
    off = synth.offsets_from_sizes([30_000, 10])
    ctx = dgs.Context(off, W=2)
    srv = Server(ctx, None, density_max=0.01)
    diff_ref = np.zeros((2, int(off[-1])), np.float32)
    wi, wv = oracle.server_pull(diff_ref, 1, off, 0.01)
    gi, gv = srv.pull(1, 0.01)
    assert_pairs_match(gi, gv, wi, wv, "empty pull")
    idx = np.array([5, 17, 29_999, 30_003], np.uint32)
    val = np.array([1.0, -2.0, 0.5, 4.0], np.float32)
    srv.push(0, idx, val)
    with pytest.raises(dgs.DgsError) as ei:
        srv.pull_all(0, capacity=3)
    assert ei.value.code == dgs.DGS_ECAPACITY
    gi, gv = srv.pull_all(0, capacity=4)
    assert list(gi) == list(idx) and list(gv) == [-1.0, 2.0, -0.5, -4.0]
    ctx.close()


def test_argument_errors(torch_mod):
    torch = torch_mod
    off = synth.offsets_from_sizes([5000, 20])
    ctx = dgs.Context(off, W=2)
    w = Worker(ctx, density_max=0.1)
    L = dgs.lib()
    h = ctx._h
    g, s, i, v = w.grad.data_ptr(), w.state.data_ptr(), w.idx.data_ptr(), w.val.data_ptr()
    assert L.dgs_worker_step(h, g, s, None, 1.0, 0.9, 0.0, i, v, None) == dgs.DGS_EINVAL      # density 0
    assert L.dgs_worker_step(h, g, s, None, 1.0, 0.9, 1.5, i, v, None) == dgs.DGS_EINVAL      # density > 1
    assert L.dgs_worker_step(h, g, s, None, 1.0, 1.0, 0.1, i, v, None) == dgs.DGS_EINVAL      # m = 1
    assert L.dgs_worker_step(h, g, None, None, 1.0, 0.5, 0.1, i, v, None) == dgs.DGS_EINVAL   # no state
    assert L.dgs_worker_step(h, g, s, s, 1.0, 0.5, 0.1, i, v, None) == dgs.DGS_ENOTSUP        # both states
    assert L.dgs_worker_step(h, g, None, s, 1.0, 0.5, 0.1, i, v, None) == dgs.DGS_EINVAL      # residual with m != 0
    assert L.dgs_worker_step(h, g, s + 2, None, 1.0, 0.5, 0.1, i, v, None) == dgs.DGS_EINVAL  # misaligned
    assert L.dgs_server_pull(h, 0, 0.1, i, v, None) == dgs.DGS_EINVAL                         # not attached
    srv = Server(ctx, None, density_max=0.1)
    assert L.dgs_server_pull(h, 2, 0.1, i, v, None) == dgs.DGS_EINVAL                         # worker id
    assert L.dgs_server_push(h, None, 5, i, v, 1) == dgs.DGS_EINVAL
    ctx.set_option(dgs.OPT_VALIDATE, 1)
    bad = to_dev(np.array([7, 7, 9], np.uint32))
    vals = to_dev(np.ones(3, np.float32))
    assert L.dgs_server_push(h, None, 0, bad.data_ptr(), vals.data_ptr(), 3) == dgs.DGS_EINVAL   # duplicate
    bad = to_dev(np.array([7, 8, 6000], np.uint32))
    assert L.dgs_server_push(h, None, 0, bad.data_ptr(), vals.data_ptr(), 3) == dgs.DGS_EINVAL   # range
    torch.cuda.synchronize()
    assert not srv.diff.any().item()
    with pytest.raises(dgs.DgsError):
        ctx.set_option(99, 1)
    ctx.close()


def test_checkpoint_resume_is_bit_identical(oracle, torch_mod):
    """All state is in caller-owned buffers; the context's threshold hints only
    steer the code path.  10 steps == 5 steps + fresh context + 5 steps."""
    torch = torch_mod
    off = synth.offsets_from_sizes([150_000, 300, 20_000])
    n = int(off[-1])
    rng = np.random.default_rng(34)
    grads = [synth.gaussian(n, rng) for _ in range(10)]
    ctx = dgs.Context(off, W=0)
    w = Worker(ctx, density_max=0.002)
    full = [w.step(g, 0.2, 0.9, 0.002) for g in grads]
    final = w.state_host()
    ctx.close()
    ctx = dgs.Context(off, W=0)
    w = Worker(ctx, density_max=0.002)
    for g in grads[:5]:
        w.step(g, 0.2, 0.9, 0.002)
    saved = w.state_host()
    ctx.close()
    ctx = dgs.Context(off, W=0)
    w = Worker(ctx, density_max=0.002)
    w.state.copy_(torch.from_numpy(saved))
    for t, g in enumerate(grads[5:]):
        i, v = w.step(g, 0.2, 0.9, 0.002)
        assert np.array_equal(i, full[5 + t][0])
        assert np.array_equal(v.view(np.uint32), full[5 + t][1].view(np.uint32))
    assert np.array_equal(w.state_host().view(np.uint32), final.view(np.uint32))
    ctx.close()


def test_repeated_pulls_without_pushes(oracle, torch_mod):
    """Pulls that find fewer nonzeros than k: zero-valued entries at the lowest indices
    complete each message (also -0.0, which keeps its sign bit in the message).  After
    the threshold hint has dropped to 'every nonzero', no dense re-selection is needed."""
    sizes = [90_000, 64, 20_000, 150_001]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    scales = synth.tensor_scales(len(sizes), 35)
    rng = np.random.default_rng(36)
    kj, K = oracle.nnz(off, 0.002)
    ctx = dgs.Context(off, W=2)
    srv = Server(ctx, None, density_max=0.01)
    diff_ref = np.zeros((2, n), np.float32)
    # a few negative zeros inside the leading run of the first tensor
    import torch
    diff_ref[0, [3, 11, 95_000]] = np.float32(-0.0)
    srv.diff.copy_(torch.from_numpy(diff_ref))
    idx, val = synth.sparse_payload(off, kj, scales, rng)
    oracle.server_push(None, diff_ref, idx, val)
    srv.push(0, idx, val)
    fallbacks = []
    for t in range(6):
        rho = 0.002 if t < 2 else 0.004        # more than was pushed
        wi, wv = oracle.server_pull(diff_ref, 0, off, rho)
        gi, gv = srv.pull(0, rho)
        assert np.array_equal(gi, wi), f"pull {t}"
        assert np.array_equal(gv.view(np.uint32), wv.view(np.uint32)), f"pull {t}"
        fallbacks.append(ctx.stats().fallback_tensors)
    assert_state_match(srv.diff.cpu().numpy()[0], diff_ref[0], "diff row 0")
    assert fallbacks[-1] == fallbacks[-3], "later empty pulls must not re-select densely"
    assert ctx.stats().internal_errors == 0
    ctx.close()


def test_density_schedule_beyond_the_plan_cache(oracle, torch_mod):
    """A warm-up style schedule over 12 densities, walked twice (more than the 8 launch plans the
    context keeps, so plans are evicted and rebuilt), then a few steps at the last one (the
    prediction takes over again); worker and pull both follow it."""
    off = synth.offsets_from_sizes(RAGGED_SIZES)
    n = int(off[-1])
    scales = synth.tensor_scales(len(RAGGED_SIZES), 30)
    rng = np.random.default_rng(31)
    schedule = [0.25, 0.125, 0.0625, 0.04, 0.03, 0.02, 0.01, 0.007, 0.004, 0.002, 0.001, 0.0005]
    ctx = dgs.Context(off, W=1)
    w = Worker(ctx, density_max=0.25)
    srv = Server(ctx, np.zeros(n, np.float32), density_max=0.25)
    s_ref = np.zeros(n, np.float32)
    model_ref = np.zeros(n, np.float32)
    diff_ref = np.zeros((1, n), np.float32)
    for t, rho in enumerate(schedule + schedule + [schedule[-1]] * 3):
        g = synth.gaussian_grads(off, scales, rng)
        wi, wv = oracle.worker_step(g, s_ref, off, np.float32(0.5), np.float32(0.9), rho)
        gi, gv = w.step(g, 0.5, 0.9, rho)
        assert_pairs_match(gi, gv, wi, wv, f"step {t} density {rho}")
        oracle.server_push(model_ref, diff_ref, wi, wv)
        ctx.server_push(srv.model, 0, w.idx, w.val, gi.size)
        pi_ref, pv_ref = oracle.server_pull(diff_ref, 0, off, rho)
        pi, pv = srv.pull(0, rho)
        assert_pairs_match(pi, pv, pi_ref, pv_ref, f"pull {t} density {rho}")
    assert_state_match(w.state_host(), s_ref, "worker state")
    assert_state_match(srv.diff.cpu().numpy()[0], diff_ref[0], "difference row")
    st = ctx.stats()
    assert st.internal_errors == 0
    assert st.exact_calls <= 2 * (2 * len(schedule) + 1)      # the last three steps are predicted
    ctx.close()


@pytest.mark.parametrize("sign", [-1.0, 0.5])
def test_apply_sparse_sign_and_range(oracle, torch_mod, sign):
    """dgs_apply_sparse (Algorithm 1/3 apply line; Eq. 5 has sign +1) with other signs: one fma
    per named entry, everything else untouched; an index outside the buffer is skipped, and
    refused before anything is written when validation is on."""
    torch = torch_mod
    rng = np.random.default_rng(77)
    sizes = [5000, 70_001, 1234]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    ctx = dgs.Context(off, W=0)
    theta0 = rng.standard_normal(n).astype(np.float32)
    idx = np.sort(rng.choice(n, 3000, replace=False)).astype(np.uint32)
    val = rng.standard_normal(3000).astype(np.float32)
    val[:50] = theta0[idx[:50]] * np.float32(1.0 + 2.0 ** -20)
    want = theta0.copy()
    oracle.apply_sparse(want, idx, val, sign)
    theta = to_dev(theta0)
    ctx.apply_sparse(theta, to_dev(idx), to_dev(val), idx.size, sign)
    torch.cuda.synchronize()
    assert_state_match(theta.cpu().numpy(), want, f"apply sign {sign}")
    # a corrupted message: one index past the end
    bad = idx.copy()
    bad[-1] = n + 5
    want2 = want.copy()
    oracle.apply_sparse(want2, idx[:-1], val[:-1], sign)
    guard = torch.zeros(n + 64, dtype=torch.float32, device="cuda:0")
    guard[:n].copy_(theta)
    ctx.apply_sparse(guard[:n], to_dev(bad), to_dev(val), bad.size, sign)
    torch.cuda.synchronize()
    assert_state_match(guard[:n].cpu().numpy(), want2, "out-of-range entry skipped")
    assert not guard[n:].any().item(), "write past the destination"
    ctx.set_option(dgs.OPT_VALIDATE, 1)
    before = guard.clone()
    with pytest.raises(dgs.DgsError) as ei:
        ctx.apply_sparse(guard[:n], to_dev(bad), to_dev(val), bad.size, sign)
    assert ei.value.code == dgs.DGS_EINVAL
    torch.cuda.synchronize()
    assert torch.equal(guard, before)
    ctx.close()
