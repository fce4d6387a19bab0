"""Pins for the CPU oracle: everything here checks `oracle/` against something
other than itself -- identities the paper states, closed forms, exact rational
arithmetic, brute force, literal re-statements of Algorithms 1-3 in numpy, and
a hand-worked example.  No GPU.
"""
import json
import os
import re
from fractions import Fraction

import numpy as np
import pytest

from paper_1910_10929_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


# ----------------------------------------------------------------------------
# independent helpers (none of them calls the oracle)
# ----------------------------------------------------------------------------

def key_of(x: np.ndarray) -> np.ndarray:
    return x.view(np.uint32) & np.uint32(0x7FFFFFFF)


def topk_numpy(a: np.ndarray, k: int) -> np.ndarray:
    """k largest magnitudes, ties to the lower index, ascending positions."""
    key = key_of(a).astype(np.int64)
    order = np.lexsort((np.arange(a.size), -key))
    return np.sort(order[:k]).astype(np.uint32)


def round_fraction_to_f32(x: Fraction) -> np.float32:
    """Round an exact rational to the nearest binary32 (ties to even), keeping
    subnormals.  Integer arithmetic only."""
    if x == 0:
        return np.float32(0.0)
    sign = -1 if x < 0 else 1
    x = abs(x)
    e = x.numerator.bit_length() - x.denominator.bit_length()
    if Fraction(2) ** e > x:
        e -= 1
    assert Fraction(2) ** e <= x < Fraction(2) ** (e + 1)
    qexp = max(e, -126) - 23                       # exponent of one ulp
    q = x / (Fraction(2) ** qexp)
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (fl & 1)):
        fl += 1
    return np.float32(sign * float(fl) * (2.0 ** qexp))


def exact_fma_f32(lr, g, s):
    return round_fraction_to_f32(Fraction(float(lr)) * Fraction(float(g)) + Fraction(float(s)))


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32)


def ceil_rho_n(density: float, n: int) -> int:
    """ceil(density * n) with the product rounded to double, by exact
    arithmetic."""
    prod = float(Fraction(density) * n)   # Fraction -> float is correctly rounded
    f = Fraction(prod)
    return -((-f.numerator) // f.denominator)


# ----------------------------------------------------------------------------
# k = ceil(rho * n) and nnz
# ----------------------------------------------------------------------------

def test_k_values(oracle):
    assert oracle.k_of(0.01, 1 << 20) == 10486
    assert oracle.k_of(1.0, 77) == 77
    assert oracle.k_of(0.001, 64) == 1
    assert oracle.k_of(0.25, 8) == 2
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(1, 1 << 31))
        rho = float(rng.choice([1e-4, 1e-3, 1e-2, 0.1, 0.3, 0.5, 1.0, rng.random() + 1e-9]))
        assert oracle.k_of(rho, n) == ceil_rho_n(rho, n)


def test_resnet50_layout_and_nnz(oracle):
    off = synth.layout_resnet50()
    assert len(off) - 1 == 161
    assert int(off[-1]) == 25_557_032
    kj, K = oracle.nnz(off, 1e-3)
    assert K == 25_670
    assert kj.min() >= 1
    off4 = synth.layout_transformer()
    assert len(off4) - 1 == 49 and int(off4[-1]) == 108_375_552
    assert oracle.nnz(off4, 1e-3)[1] == 108_401
    off5 = synth.layout_equal(1_000_000_000, 64)
    assert oracle.nnz(off5, 1e-4)[1] == 100_032
    assert oracle.nnz(off5, 1e-2)[1] == 10_000_000


# ----------------------------------------------------------------------------
# selection: brute force, numpy definition, adversarial ties
# ----------------------------------------------------------------------------

def _tie_cases():
    rng = np.random.default_rng(11)
    cases = []
    cases.append(("all_equal", np.full(37, 2.5, np.float32)))
    cases.append(("all_zero", np.zeros(29, np.float32)))
    cases.append(("pm_pairs", np.array([1, -1, 2, -2, 3, -3, 3, -3, 0.5, -0.5], np.float32)))
    cases.append(("neg_zero", np.array([0.0, -0.0, 0.0, 1e-40, -0.0, 0.0], np.float32)))
    cases.append(("single", np.array([-7.0], np.float32)))
    cases.append(("few_levels", rng.integers(-3, 4, size=257).astype(np.float32)))
    cases.append(("gauss", rng.standard_normal(1000).astype(np.float32)))
    cases.append(("mostly_zero", (rng.standard_normal(512) * (rng.random(512) < 0.05)).astype(np.float32)))
    cases.append(("inf_nan", np.array([1.0, np.inf, -np.inf, np.nan, 3.0, -2.0], np.float32)))
    cases.append(("denormals", (rng.integers(-50, 50, size=64).astype(np.float32) * np.float32(1e-45))))
    return cases


@pytest.mark.parametrize("name,a", _tie_cases(), ids=[c[0] for c in _tie_cases()])
def test_selection_against_bruteforce_and_numpy(oracle, name, a):
    n = a.size
    for k in sorted({1, 2, 3, n // 3, n // 2, n - 1, n} - {0}):
        if k < 1 or k > n:
            continue
        want = topk_numpy(a, k)
        got = oracle.topk(a, k)
        brute = oracle.topk_bruteforce(a, k)
        assert np.array_equal(got, want), (name, k)
        assert np.array_equal(brute, want), (name, k)


def test_selection_random_small(oracle):
    rng = np.random.default_rng(2)
    for trial in range(300):
        n = int(rng.integers(1, 200))
        levels = int(rng.integers(1, 6))
        a = rng.integers(-levels, levels + 1, size=n).astype(np.float32)
        if trial % 3 == 0:
            a = rng.standard_normal(n).astype(np.float32)
        k = int(rng.integers(1, n + 1))
        assert np.array_equal(oracle.topk(a, k), topk_numpy(a, k))
        assert np.array_equal(oracle.topk_bruteforce(a, k), topk_numpy(a, k))


def test_ordering_of_specials(oracle):
    # NaN > Inf > finite in magnitude-key order; sign is ignored
    a = np.array([5.0, -np.inf, np.nan, 1e30, np.inf], np.float32)
    assert list(oracle.topk(a, 1)) == [2]
    assert list(oracle.topk(a, 3)) == [1, 2, 4]


# ----------------------------------------------------------------------------
# worker step
# ----------------------------------------------------------------------------

def test_fma_is_single_rounding(oracle):
    """a = fmaf(lr, g, s) must equal the exactly rounded lr*g + s (Algorithm 3,
    accumulate step), including cases where mul-then-add differs."""
    rng = np.random.default_rng(3)
    n = 400
    g = rng.standard_normal(n).astype(np.float32)
    s = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g[:8] = np.float32(1.0) + np.float32(2.0 ** -23) * np.arange(1, 9, dtype=np.float32)
    s[:8] = -g[:8] * g[:8]                      # catastrophic cancellation cases
    g[8:12] = np.array([1e-40, -3e-42, 2e-45, 1e-38], np.float32)   # subnormal inputs
    s[8:12] = np.array([1e-41, 1e-45, -1e-45, -1e-38], np.float32)
    lr = np.float32(1.0) + np.float32(2.0 ** -23) * np.float32(3)
    off = synth.layout_flat(n)
    state = s.copy()
    idx, val = oracle.worker_step(g, state, off, float(lr), 0.0, 1.0)   # density 1: everything sent
    assert np.array_equal(idx, np.arange(n, dtype=np.uint32))
    want = np.array([exact_fma_f32(lr, g[i], s[i]) for i in range(n)], np.float32)
    assert np.array_equal(val.view(np.uint32), want.view(np.uint32))
    two_step = (lr * g + s).astype(np.float32)
    assert np.any(two_step.view(np.uint32) != want.view(np.uint32)), "test has no discriminating case"
    assert np.any((want != 0) & (np.abs(want) < np.float32(1.1754944e-38))), "no subnormal result covered"


def test_conservation_and_structure(oracle):
    """Sent + kept == accumulated, bitwise; nnz == sum_j ceil(rho n_j); ascending
    indices; exactly k_j per tensor (Algorithm 3 split step)."""
    rng = np.random.default_rng(4)
    sizes = [1, 7, 64, 333, 1000, 4096, 50]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    scales = synth.tensor_scales(len(sizes), 9)
    s = np.zeros(n, np.float32)
    m, lr, rho = np.float32(0.9), np.float32(0.5), 0.03
    for step in range(6):
        g = synth.gaussian_grads(off, scales, rng)
        a = np.array([exact_fma_f32(lr, g[i], s[i]) for i in range(n)], np.float32) if step < 2 \
            else (np.float64(lr) * g.astype(np.float64) + s.astype(np.float64)).astype(np.float32)
        s_new = s.copy()
        idx, val = oracle.worker_step(g, s_new, off, float(lr), float(m), rho)
        kj = [ceil_rho_n(rho, sz) for sz in sizes]
        assert idx.size == sum(kj)
        assert np.all(np.diff(idx.astype(np.int64)) > 0)
        for j, sz in enumerate(sizes):
            inside = (idx >= off[j]) & (idx < off[j + 1])
            assert inside.sum() == kj[j]
            want = topk_numpy(a[int(off[j]):int(off[j + 1])], kj[j]) + np.uint32(off[j])
            assert np.array_equal(idx[inside], want)
        if step < 2:
            sel = np.zeros(n, bool)
            sel[idx] = True
            assert np.array_equal(val.view(np.uint32), a[idx].view(np.uint32))
            assert np.array_equal(s_new[~sel].view(np.uint32), a[~sel].view(np.uint32))
            assert np.array_equal(s_new[sel].view(np.uint32), (m * a[sel]).view(np.uint32))
        s = s_new


def test_density_one_is_momentum_sgd(oracle):
    """With nothing dropped, the sent values are Eq. 7's velocity u_t = m u_{t-1}
    + eta grad_t and, through push + full pull + apply, theta follows theta -= u_t
    (Eq. 5, Eq. 7-8)."""
    rng = np.random.default_rng(6)
    n, m, lr = 96, 0.5, 0.25          # powers of two: every operation below is exact
    off = synth.layout_flat(n)
    state = np.zeros(n, np.float32)
    u = [0.0] * n                      # scalar reference loop
    theta_ref = [float(i) for i in range(n)]
    theta = np.arange(n, dtype=np.float32)
    model = theta.copy()
    diff = np.zeros((1, n), np.float32)
    for t in range(5):
        g = synth.integer_grads(n, rng)
        idx, val = oracle.worker_step(g, state, off, lr, m, 1.0)
        for i in range(n):
            u[i] = m * u[i] + lr * float(g[i])
            theta_ref[i] -= u[i]
        assert np.array_equal(val, np.array(u, np.float32))
        oracle.server_push(model, diff, idx, val)
        gi, gv = oracle.server_pull(diff, 0, off, 1.0)
        oracle.apply_sparse(theta, gi, gv, 1.0)
        assert np.array_equal(theta, np.array(theta_ref, np.float32))
        assert np.array_equal(model, theta)
        assert not diff.any()


def test_telescoping_over_unsent_interval(oracle):
    """Eq. 13: an entry sent at step c and next at c+T carries
    m*u_c + eta * (sum of the T gradients in between), exactly."""
    rng = np.random.default_rng(7)
    n, m, lr = 512, 0.5, 1.0
    off = synth.layout_flat(n)
    state = np.zeros(n, np.float32)
    last_sent_u = np.zeros(n, np.float64)       # u at the last send (0 before any send)
    acc = np.zeros(n, np.float64)               # sum of grads since the last send
    checked = 0
    for t in range(12):
        g = synth.integer_grads(n, rng, -4, 4)
        acc += g
        idx, val = oracle.worker_step(g, state, off, lr, m, 0.05)
        want = m * last_sent_u[idx] + lr * acc[idx]
        assert np.array_equal(val.astype(np.float64), want)
        checked += idx.size
        last_sent_u[idx] = val
        acc[idx] = 0.0
    assert checked > 100


def alg1_literal(g, v, off, lr, rho, kfun):
    """Algorithm 1 written out in numpy (residual accumulation, top-k mask,
    send masked, keep the rest), with the mask applied to the un-masked v."""
    v = (v + lr * g).astype(np.float32)
    out_i, out_v = [], []
    for j in range(len(off) - 1):
        a, b = int(off[j]), int(off[j + 1])
        pick = topk_numpy(v[a:b], kfun(rho, b - a)) + a
        out_i.append(pick)
        out_v.append(v[pick].copy())
        v[pick] = 0.0
    return v, np.concatenate(out_i).astype(np.uint32), np.concatenate(out_v)


def test_momentum_zero_is_algorithm_1(oracle):
    rng = np.random.default_rng(8)
    sizes = [300, 17, 1024]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    v = np.zeros(n, np.float32)
    s = np.zeros(n, np.float32)
    for t in range(8):
        g = synth.integer_grads(n, rng)          # lr = 0.5, integers: mul+add is exact, so fma == mul-add
        v, wi, wv = alg1_literal(g, v, off, np.float32(0.5), 0.02, ceil_rho_n)
        idx, val = oracle.worker_step(g, s, off, 0.5, 0.0, 0.02)
        assert np.array_equal(idx, wi)
        assert np.array_equal(val, wv)
        assert np.array_equal(s.view(np.uint32) & 0x7FFFFFFF, v.view(np.uint32) & 0x7FFFFFFF)
        assert np.array_equal(s, v)


def alg3_literal_u(g, u, off, lr, m, rho, kfun):
    """Algorithm 3 as printed: u <- m u + eta g; per tensor mask by top-k of |u|;
    send u*Mask; u <- u + (1/m - 1) * u * notMask."""
    u = (np.float32(m) * u + np.float32(lr) * g).astype(np.float32)
    out_i, out_v = [], []
    mask = np.zeros(u.size, bool)
    for j in range(len(off) - 1):
        a, b = int(off[j]), int(off[j + 1])
        pick = topk_numpy(u[a:b], kfun(rho, b - a)) + a
        out_i.append(pick)
        out_v.append(u[pick].copy())
        mask[pick] = True
    scale = np.float32(1.0 / m - 1.0)
    u = np.where(mask, u, (u + scale * u).astype(np.float32)).astype(np.float32)
    return u, np.concatenate(out_i).astype(np.uint32), np.concatenate(out_v)


def test_against_literal_algorithm_3_exact_inputs(oracle):
    """With m = 0.5, lr = 1 and integer gradients every operation is exact in
    fp32, so the s = m*u storage must agree bitwise with the printed u-form."""
    rng = np.random.default_rng(9)
    sizes = [513, 64, 2000]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    u = np.zeros(n, np.float32)
    s = np.zeros(n, np.float32)
    for t in range(10):
        g = synth.integer_grads(n, rng, -6, 6)
        u, wi, wv = alg3_literal_u(g, u, off, 1.0, 0.5, 0.01, ceil_rho_n)
        idx, val = oracle.worker_step(g, s, off, 1.0, 0.5, 0.01)
        assert np.array_equal(idx, wi), t
        assert np.array_equal(val, wv), t
        assert np.array_equal(s, np.float32(0.5) * u), t


def test_against_literal_algorithm_3_gaussian(oracle):
    """General inputs: the printed form rounds differently (1/m rescale, no fma),
    so indices agree on the first step and values stay within 1e-5 relative."""
    rng = np.random.default_rng(10)
    off = synth.offsets_from_sizes([4096, 1000])
    n = int(off[-1])
    u = np.zeros(n, np.float32)
    s = np.zeros(n, np.float32)
    for t in range(10):
        g = synth.gaussian(n, rng)
        u, wi, wv = alg3_literal_u(g, u, off, 0.1, 0.9, 0.01, ceil_rho_n)
        idx, val = oracle.worker_step(g, s, off, np.float32(0.1), np.float32(0.9), 0.01)
        if t == 0:
            assert np.array_equal(idx, wi)
        common = np.intersect1d(idx, wi)
        assert common.size >= 0.9 * idx.size
        lookup_a = dict(zip(idx.tolist(), val.tolist()))
        lookup_b = dict(zip(wi.tolist(), wv.tolist()))
        for i in common[:200]:
            assert abs(lookup_a[i] - lookup_b[i]) <= 1e-5 * abs(lookup_b[i]) + 1e-9
        np.testing.assert_allclose(s, np.float32(0.9) * u, rtol=2e-5, atol=2e-7)  # cancellation near 0


# ----------------------------------------------------------------------------
# server
# ----------------------------------------------------------------------------

def alg2_literal_v(M, v_k, idx, val, off, rho, kfun):
    """Algorithm 2 as printed, dense: M <- M - decode(g); G = M - v_k; per tensor
    keep top-k of |G|; v_k <- v_k + G (the sign that Eq. 4 / Eq. 6 require)."""
    M = M.copy()
    M[idx] = M[idx] - val
    G = (M - v_k).astype(np.float32)
    out_i, out_v = [], []
    for j in range(len(off) - 1):
        a, b = int(off[j]), int(off[j + 1])
        pick = topk_numpy(G[a:b], kfun(rho, b - a)) + a
        out_i.append(pick)
        out_v.append(G[pick].copy())
    gi = np.concatenate(out_i).astype(np.uint32)
    gv = np.concatenate(out_v)
    v_k = v_k.copy()
    v_k[gi] = v_k[gi] + gv
    return M, v_k, gi, gv


def test_server_against_literal_algorithm_2_and_identities(oracle):
    """Integer data (exact arithmetic).  Checks: the D-form equals the printed
    v-form (Algorithm 2, Eq. 6); M == -sum of pushes (Eq. 1); theta_k + D_k ==
    theta_0 + M at all times (Eq. 2-5); a full pull empties D_k (DGS without
    sparsification == ASGD)."""
    rng = np.random.default_rng(12)
    sizes = [400, 33, 1200]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    W = 4
    rho_up, rho_down = 0.05, 0.02
    theta0 = rng.integers(-5, 6, size=n).astype(np.float32)
    model = theta0.copy()
    diff = np.zeros((W, n), np.float32)
    theta_k = [theta0.copy() for _ in range(W)]
    M_lit = np.zeros(n, np.float32)
    v_lit = [np.zeros(n, np.float32) for _ in range(W)]
    pushed_sum = np.zeros(n, np.float64)
    kj = [ceil_rho_n(rho_up, s) for s in sizes]
    order = synth.event_schedule(W, 40, 3)
    for e, k in enumerate(order):
        k = int(k)
        idx, val = synth.sparse_payload(off, kj, None, rng)
        val = np.round(val * 4).astype(np.float32)
        oracle.server_push(model, diff, idx, val)
        pushed_sum[idx] += val
        M_lit, v_lit[k], wi, wv = alg2_literal_v(M_lit, v_lit[k], idx, val, off, rho_down, ceil_rho_n)
        gi, gv = oracle.server_pull(diff, k, off, rho_down)
        assert np.array_equal(gi, wi), e
        assert np.array_equal(gv, wv), e
        oracle.apply_sparse(theta_k[k], gi, gv, 1.0)
        assert np.array_equal((model - theta0).astype(np.float64), -pushed_sum)
        assert np.array_equal(M_lit, model - theta0)
        for w in range(W):
            assert np.array_equal(theta_k[w] + diff[w], model)
            assert np.array_equal(diff[w], M_lit - v_lit[w])
    for w in range(W):
        gi, gv = oracle.server_pull(diff, w, off, 1.0)
        assert gi.size == n
        oracle.apply_sparse(theta_k[w], gi, gv, 1.0)
        assert not diff[w].any()
        assert np.array_equal(theta_k[w], model)


def test_printed_server_form_against_literal_algorithm_2(oracle):
    """The oracle's model / sent_k form (Algorithm 2 as printed) against the dense numpy
    statement above, on Gaussian data (same fp32 operations, so bit equality), and
    against the difference-row form on integer data, where both are exact."""
    rng = np.random.default_rng(14)
    sizes = [700, 5, 1300]
    off = synth.offsets_from_sizes(sizes)
    n = int(off[-1])
    W = 3
    rho_up, rho_down = 0.03, 0.02
    kj = [ceil_rho_n(rho_up, s) for s in sizes]
    order = synth.event_schedule(W, 30, 15)
    # Gaussian values, theta_0 = 0: M and v_k of the printed algorithm are model and sent_k
    model = np.zeros(n, np.float32)
    sent = np.zeros((W, n), np.float32)
    M_lit = np.zeros(n, np.float32)
    v_lit = [np.zeros(n, np.float32) for _ in range(W)]
    for e, k in enumerate(order):
        k = int(k)
        idx, val = synth.sparse_payload(off, kj, None, rng)
        oracle.server_push_model(model, idx, val)
        M_lit, v_lit[k], wi, wv = alg2_literal_v(M_lit, v_lit[k], idx, val, off, rho_down, ceil_rho_n)
        gi, gv = oracle.server_pull_sent(model, sent, k, off, rho_down)
        assert np.array_equal(gi, wi), e
        assert np.array_equal(bits(gv), bits(wv)), e
        assert np.array_equal(bits(model), bits(M_lit))
        assert np.array_equal(bits(sent[k]), bits(v_lit[k]))
    # integer data, theta_0 != 0: identical messages from both server forms
    theta0 = rng.integers(-5, 6, size=n).astype(np.float32)
    model_d, model_s = theta0.copy(), theta0.copy()
    diff = np.zeros((W, n), np.float32)
    sent = np.tile(theta0, (W, 1))
    for e, k in enumerate(order):
        k = int(k)
        idx, val = synth.sparse_payload(off, kj, None, rng)
        val = np.round(val * 4).astype(np.float32)
        oracle.server_push(model_d, diff, idx, val)
        oracle.server_push_model(model_s, idx, val)
        di, dv = oracle.server_pull(diff, k, off, rho_down)
        si, sv = oracle.server_pull_sent(model_s, sent, k, off, rho_down)
        assert np.array_equal(di, si) and np.array_equal(dv, sv), e
        assert np.array_equal(model_d, model_s)
        for w in range(W):
            assert np.array_equal(diff[w], model_s - sent[w])
    # density 1: the worker is brought fully up to date (sent_k == model)
    for w in range(W):
        oracle.server_pull_sent(model_s, sent, w, off, 1.0)
        assert np.array_equal(sent[w], model_s)


def test_printed_server_form_without_secondary_compression(oracle):
    """Algorithm 2 with the compression switch off on the printed state: G = M - v_k whole
    (Eq. 3), v_k += G (Eq. 6).  Against the dense numpy statement on Gaussian data (bits),
    against the difference-row form on integer data (both exact), and v_k == M afterwards."""
    rng = np.random.default_rng(16)
    n, W = 3000, 3
    off = synth.layout_flat(n)
    order = synth.event_schedule(W, 20, 17)
    model = rng.standard_normal(n).astype(np.float32)
    sent = np.tile(model, (W, 1))
    for e, k in enumerate(order):
        k = int(k)
        idx, val = synth.sparse_payload(off, [40], None, rng)
        oracle.server_push_model(model, idx, val)
        G = model - sent[k]                                    # dense, fp32
        nz = np.nonzero(key_of(G))[0]
        want_sent = sent[k].copy()
        want_sent[nz] = want_sent[nz] + G[nz]
        gi, gv = oracle.server_pull_all_sent(model, sent, k)
        assert np.array_equal(gi, nz.astype(np.uint32)), e
        assert np.array_equal(bits(gv), bits(G[nz])), e
        assert np.array_equal(bits(sent[k]), bits(want_sent)), e
    theta0 = rng.integers(-5, 6, size=n).astype(np.float32)
    model_d, model_s = theta0.copy(), theta0.copy()
    diff = np.zeros((W, n), np.float32)
    sent = np.tile(theta0, (W, 1))
    for e, k in enumerate(order):
        k = int(k)
        idx, val = synth.sparse_payload(off, [40], None, rng)
        val = np.round(val * 4).astype(np.float32)
        oracle.server_push(model_d, diff, idx, val)
        oracle.server_push_model(model_s, idx, val)
        di, dv = oracle.server_pull_all(diff, k)
        si, sv = oracle.server_pull_all_sent(model_s, sent, k)
        assert np.array_equal(di, si) and np.array_equal(dv, sv), e
        assert np.array_equal(sent[k], model_s)
    # capacity: three nonzeros do not fit two slots; the refused call changes nothing
    oracle.server_push_model(model_s, np.array([1, 2, 3], np.uint32), np.ones(3, np.float32))
    before = sent[0].copy()
    with pytest.raises(Exception):
        oracle.server_pull_all_sent(model_s, sent, 0, capacity=2)
    assert np.array_equal(bits(sent[0]), bits(before))
    gi, gv = oracle.server_pull_all_sent(model_s, sent, 0, capacity=3)   # exactly enough
    assert np.array_equal(gi, np.array([1, 2, 3], np.uint32)) and np.array_equal(gv, -np.ones(3, np.float32))


def test_double_pull_returns_next_k(oracle):
    rng = np.random.default_rng(13)
    off = synth.offsets_from_sizes([1000, 500])
    n = int(off[-1])
    diff = np.zeros((1, n), np.float32)
    diff[0] = rng.permutation(n).astype(np.float32) - n / 2 + 0.25     # distinct magnitudes
    original = diff[0].copy()
    i1, v1 = oracle.server_pull(diff, 0, off, 0.01)
    i2, v2 = oracle.server_pull(diff, 0, off, 0.01)
    both = np.sort(np.concatenate([i1, i2]))
    want = np.concatenate([topk_numpy(original[:1000], 20), topk_numpy(original[1000:], 10) + 1000])
    assert np.array_equal(both, want)
    assert np.array_equal(original[i2], v2)
    assert np.intersect1d(i1, i2).size == 0


def test_pull_with_fewer_than_k_nonzeros_emits_lowest_index_zeros(oracle):
    off = synth.layout_flat(100)
    diff = np.zeros((1, 100), np.float32)
    diff[0, [40, 70]] = [3.0, -1.0]
    idx, val = oracle.server_pull(diff, 0, off, 0.05)      # k = 5
    assert list(idx) == [0, 1, 2, 40, 70]
    assert list(val) == [0.0, 0.0, 0.0, 3.0, -1.0]
    assert not diff.any()


def test_pull_all_without_secondary_compression(oracle):
    rng = np.random.default_rng(14)
    n = 300
    diff = np.zeros((2, n), np.float32)
    pos = np.sort(rng.choice(n, 25, replace=False))
    diff[1, pos] = rng.standard_normal(25).astype(np.float32)
    diff[1, pos[3]] = -0.0
    want_pos = np.delete(pos, 3)
    want_val = diff[1, want_pos].copy()
    idx, val = oracle.server_pull_all(diff, 1)
    assert np.array_equal(idx, want_pos.astype(np.uint32))
    assert np.array_equal(val, want_val)
    assert not diff[1].any()


def test_pull_all_capacity_branch(oracle):
    """Algorithm 2 with the compression switch off, on the difference rows: a message that
    does not fit `capacity` is refused, the count is still reported, and the row is left
    as it was; with exactly enough room it goes through."""
    n = 64
    diff = np.zeros((1, n), np.float32)
    pos = np.array([3, 9, 10, 40, 63])
    diff[0, pos] = np.array([1.5, -2.0, 1e-40, -0.25, 7.0], np.float32)   # one subnormal: still nonzero
    before = diff[0].copy()
    lib = oracle.lib()
    import ctypes
    idx = np.zeros(8, np.uint32)
    val = np.zeros(8, np.float32)
    cnt = ctypes.c_uint64(0)
    f32p, u32p = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint32)
    rc = lib.dgs_oracle_server_pull_all(diff[0].ctypes.data_as(f32p), n, idx.ctypes.data_as(u32p),
                                        val.ctypes.data_as(f32p), 4, ctypes.byref(cnt))
    assert rc != 0 and cnt.value == 5
    assert np.array_equal(bits(diff[0]), bits(before)) and not idx.any() and not val.any()
    with pytest.raises(Exception):
        oracle.server_pull_all(diff, 0, capacity=4)
    gi, gv = oracle.server_pull_all(diff, 0, capacity=5)
    assert np.array_equal(gi, pos.astype(np.uint32)) and np.array_equal(bits(gv), bits(before[pos]))
    assert not diff[0].any()


@pytest.mark.parametrize("sign", [1.0, -1.0, 0.5, -0.333251953125])
def test_apply_sparse_is_one_fma_with_the_sign(oracle, sign):
    """Worker applies decode(G): theta[idx] = fma(sign, val, theta[idx]) (Eq. 5 has sign +1),
    against exact rational arithmetic; entries not named stay untouched."""
    rng = np.random.default_rng(21)
    n = 300
    theta = rng.standard_normal(n).astype(np.float32)
    idx = np.sort(rng.choice(n, 120, replace=False)).astype(np.uint32)
    val = rng.standard_normal(120).astype(np.float32)
    val[:6] = theta[idx[:6]] * np.float32(1.0 + 2.0 ** -20)      # near-cancellation when sign = -1
    val[6:9] = np.array([1e-40, -2e-45, 3e-39], np.float32)      # subnormal values
    theta[idx[6:9]] = np.array([-1e-41, 1e-45, 1e-38], np.float32)
    want = theta.copy()
    for e, i in enumerate(idx):
        want[i] = exact_fma_f32(np.float32(sign), val[e], theta[i])
    got = theta.copy()
    oracle.apply_sparse(got, idx, val, sign)
    assert np.array_equal(bits(got), bits(want))
    if sign not in (1.0, -1.0):
        two_step = theta.copy()
        two_step[idx] = (np.float32(sign) * val).astype(np.float32) + theta[idx]
        assert np.any(bits(two_step) != bits(want)), "no case separates one rounding from two"
    else:
        flipped = theta.copy()
        flipped[idx] = theta[idx] - np.float32(sign) * val
        assert np.any(bits(flipped) != bits(want)), "the sign is not observable"


def test_hand_example(oracle):
    with open(os.path.join(HERE, "golden", "x1_hand_example.json")) as f:
        ex = json.load(f)
    n = ex["n"]
    off = synth.layout_flat(n)
    s = np.array(ex["worker"][0]["state_before"], np.float32)
    for step in ex["worker"]:
        g = np.array(step["grad"], np.float32)
        idx, val = oracle.worker_step(g, s, off, ex["lr"], ex["m"], ex["density"])
        assert list(idx) == step["idx"]
        assert list(val) == step["val"]
        assert list(s) == step["state_after"]
        if "velocity_u_after" in step:
            assert list(s / np.float32(ex["m"])) == step["velocity_u_after"]
    W = ex["server"]["W"]
    model = np.zeros(n, np.float32)
    diff = np.zeros((W, n), np.float32)
    for ev in ex["server"]["events"]:
        if ev["op"] == "push":
            oracle.server_push(model, diff, np.array(ev["idx"], np.uint32), np.array(ev["val"], np.float32))
            assert list(model) == ev["model"]
        else:
            idx, val = oracle.server_pull(diff, ev["worker"], off, ex["density"])
            assert list(idx) == ev["idx"]
            assert list(val) == ev["val"]
        assert diff.tolist() == ev["diff"]


def wire_by_big_integers(off, kj, idx, val) -> bytes:
    """The wire form built with Python integers: one big integer per index block."""
    out = np.ascontiguousarray(val).astype("<f4").tobytes()
    o = 0
    for j in range(len(off) - 1):
        nj = int(off[j + 1] - off[j])
        b = max(1, (nj - 1).bit_length())
        block = 0
        for e in range(int(kj[j])):
            block |= (int(idx[o]) - int(off[j])) << (e * b)
            o += 1
        out += block.to_bytes(4 * ((int(kj[j]) * b + 31) // 32), "little")
    return out


def test_wire_form_hand_example(oracle):
    with open(os.path.join(HERE, "golden", "x2_wire_example.json")) as f:
        ex = json.load(f)
    off = synth.offsets_from_sizes(ex["sizes"])
    kj, K = oracle.nnz(off, ex["density"])
    assert list(kj) == ex["k"] and K == len(ex["idx"])
    idx = np.array(ex["idx"], np.uint32)
    val = np.array([int(h, 16) for h in ex["val_bits_hex"]], np.uint32).view(np.float32)
    want = bytes.fromhex(ex["wire_hex"].replace(" ", ""))
    assert oracle.wire_bytes(off, ex["density"]) == len(want) == 48
    assert oracle.encode(off, ex["density"], idx, val).tobytes() == want
    di, dv = oracle.decode(off, ex["density"], np.frombuffer(want, np.uint8).copy())
    assert np.array_equal(di, idx) and np.array_equal(bits(dv), bits(val))
    ex2 = ex["second"]
    off2 = synth.offsets_from_sizes(ex2["sizes"])
    val2 = np.array([int(h, 16) for h in ex2["val_bits_hex"]], np.uint32).view(np.float32)
    want2 = bytes.fromhex(ex2["wire_hex"].replace(" ", ""))
    assert oracle.encode(off2, ex2["density"], np.array(ex2["idx"], np.uint32), val2).tobytes() == want2


def test_wire_form_against_big_integer_construction(oracle):
    rng = np.random.default_rng(77)
    for trial in range(12):
        J = int(rng.integers(1, 9))
        rho = float(rng.choice([1e-3, 0.01, 0.3, 1.0]))
        pool = [1, 2, 3, 31, 32, 33, 255, 256, 257, 1000, 4096, 65_536, 65_537, 100_003, 1 << 20]
        pool = [x for x in pool if x * rho <= 4096]          # keeps the big integers small
        sizes = [int(x) for x in rng.choice(pool, J)]
        off = synth.offsets_from_sizes(sizes)
        kj, K = oracle.nnz(off, rho)
        idx = np.concatenate([np.sort(rng.choice(sizes[j], int(kj[j]), replace=False)) + int(off[j])
                              for j in range(J)]).astype(np.uint32)
        val = rng.integers(0, 1 << 32, K, dtype=np.uint64).astype(np.uint32).view(np.float32)   # any bit pattern
        want = wire_by_big_integers(off, kj, idx, val)
        assert oracle.wire_bytes(off, rho) == len(want)
        wire = oracle.encode(off, rho, idx, val)
        assert wire.tobytes() == want, f"trial {trial}: sizes {sizes} density {rho}"
        di, dv = oracle.decode(off, rho, wire)
        assert np.array_equal(di, idx) and np.array_equal(bits(dv), bits(val))


def bf16_by_rationals(b32: int) -> int:
    """Nearest bfloat16 of a finite binary32, by exact rational arithmetic: the two bfloat16
    neighbours (bit patterns with the low half cleared, as integers on the ordered line of
    magnitudes) and the distances to them as Fractions."""
    from fractions import Fraction
    sign = b32 >> 31
    mag = b32 & 0x7FFFFFFF

    def value(m):          # magnitude of the binary32 with bit pattern m (finite or the 2^128 that "inf" stands for)
        e, f = m >> 23, m & 0x7FFFFF
        if e == 0:
            return Fraction(f, 1 << 149)
        return Fraction((1 << 23) + f, 1 << 23) * (Fraction(2) ** (e - 127))
    lo = mag & 0x7FFF0000
    hi = lo + 0x10000
    v, vl, vh = value(mag), value(lo), value(hi)
    if v - vl < vh - v:
        pick = lo
    elif v - vl > vh - v:
        pick = hi
    else:
        pick = lo if ((lo >> 16) & 1) == 0 else hi
    return (sign << 15) | (pick >> 16)


def test_wire16_rounding_table_and_hand_example(oracle):
    with open(os.path.join(HERE, "golden", "x3_wire16_example.json")) as f:
        ex = json.load(f)
    off1 = synth.offsets_from_sizes([1])
    for src, want in ex["rounding"]:
        val = np.array([int(src, 16)], np.uint32).view(np.float32)
        wire = oracle.encode16(off1, 1.0, np.array([0], np.uint32), val)
        got = int(wire[0]) | (int(wire[1]) << 8)
        assert got == int(want, 16), f"{src}: {got:04X} != {want}"
        _, back = oracle.decode16(off1, 1.0, wire)
        assert int(bits(back)[0]) == int(want, 16) << 16
    m = ex["message"]
    off = synth.offsets_from_sizes(m["sizes"])
    kj, K = oracle.nnz(off, m["density"])
    assert list(kj) == m["k"]
    idx = np.array(m["idx"], np.uint32)
    val = np.array([int(h, 16) for h in m["val_bits_hex"]], np.uint32).view(np.float32)
    want = bytes.fromhex(m["wire_hex"].replace(" ", ""))
    assert oracle.wire_bytes16(off, m["density"]) == len(want) == 16
    assert oracle.encode16(off, m["density"], idx, val).tobytes() == want
    di, dv = oracle.decode16(off, m["density"], np.frombuffer(want, np.uint8).copy())
    assert np.array_equal(di, idx)
    assert [f"{int(b):08X}" for b in bits(dv)] == m["decoded_bits_hex"]


def test_wire16_against_rational_rounding_and_the_32_bit_index_blocks(oracle):
    """Random finite values (every exponent, also subnormals and halfway patterns): the value
    area against exact rational rounding, the index area byte for byte equal to the 32-bit
    form's (pinned above), the decoded value never further from the original than half a
    bfloat16 step."""
    rng = np.random.default_rng(78)
    for trial in range(20):
        sizes = [int(x) for x in rng.integers(1, 5000, size=int(rng.integers(1, 6)))]
        off = synth.offsets_from_sizes(sizes)
        rho = float(rng.choice([0.01, 0.1, 0.5, 1.0]))
        kj, K = oracle.nnz(off, rho)
        idx = np.concatenate([off[j] + np.sort(rng.choice(sizes[j], size=int(kj[j]), replace=False))
                              for j in range(len(sizes))]).astype(np.uint32)
        b32 = rng.integers(0, 1 << 32, size=K, dtype=np.uint64).astype(np.uint32)
        b32[(b32 & 0x7F800000) == 0x7F800000] &= np.uint32(0x807FFFFF)     # keep them finite
        if K > 4:
            b32[:4] = [0x3F808000, 0x3F818000, 0x00018000, 0x7F7FFFFF]
        val = b32.view(np.float32)
        wire = oracle.encode16(off, rho, idx, val)
        va = 4 * ((2 * K + 3) // 4)
        got = wire[:2 * K].view("<u2")
        want = np.array([bf16_by_rationals(int(b)) for b in b32], np.uint16)
        assert np.array_equal(got, want), f"trial {trial}"
        assert not wire[2 * K:va].any()
        assert wire[va:].tobytes() == oracle.encode(off, rho, idx, val)[4 * K:].tobytes()
        di, dv = oracle.decode16(off, rho, wire)
        assert np.array_equal(di, idx)
        assert np.array_equal(bits(dv), want.astype(np.uint32) << 16)


def test_wire_form_rejects_entries_outside_their_tensor(oracle):
    off = synth.offsets_from_sizes([10, 10])
    val = np.ones(2, np.float32)
    with pytest.raises(Exception):
        oracle.encode(off, 0.1, np.array([3, 7], np.uint32), val)        # second entry not in tensor 1
    off1 = synth.offsets_from_sizes([100])
    with pytest.raises(Exception):
        oracle.encode(off1, 0.02, np.array([5, 5], np.uint32), val)      # not ascending
    wire = oracle.encode(off1, 0.02, np.array([5, 99], np.uint32), val)
    wire[8] = 0xFF                                                       # local index 127 >= n
    with pytest.raises(Exception):
        oracle.decode(off1, 0.02, wire)


def test_oracle_sources_are_independent_of_the_product():
    """The oracle and the HIP path share no code and do not import each other."""
    root = os.path.dirname(HERE)
    for dirpath, _, files in os.walk(os.path.join(root, "oracle")):
        for fn in files:
            if fn.endswith((".c", ".h", ".py")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "paper_1910_10929_amd" not in text, fn
                assert "csrc" not in text and "dgs.h" not in text, fn
    for dirpath, _, files in os.walk(os.path.join(root, "paper_1910_10929_amd")):
        for fn in files:
            if fn.endswith((".py", ".hip", ".cpp", ".h", ".hpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "dgs_oracle" not in text, fn
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), fn
