"""Pins for the oracle's sampler: the tree recursion, the selection rules, the output definitions."""
import math
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from oracle import nuts_ref as R
from paper_1910_11141_amd import workloads as W


def target_of(w, dtype=None):
    return R.Target(w.kind, w.dim, dtype or w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y,
                    prior_scale=w.prior_scale)


def py_normals(seed, tag, iteration, chain, dim):
    """N(0,1) components for one chain, rebuilt from the draw keys with Python's own math."""
    out = []
    for k in range((dim + 1) // 2):
        w = [int(x) for x in R.draw(seed, k, tag, 0, iteration, chain)]
        u1 = (2 * (((w[0] >> 6) << 26) | (w[1] >> 6)) + 1) / 2.0**53
        u2 = (2 * (((w[2] >> 6) << 26) | (w[3] >> 6)) + 1) / 2.0**53
        rho = math.sqrt(-2.0 * math.log(u1))
        out += [rho * math.cos(2 * math.pi * u2), rho * math.sin(2 * math.pi * u2)]
    return np.array(out[:dim])


def py_u(seed, index, tag, level, iteration, chain):
    w = [int(x) for x in R.draw(seed, index, tag, level, iteration, chain)]
    return Fraction(2 * (((w[0] >> 6) << 26) | (w[1] >> 6)) + 1, 2**53)


# ------------------------------------------------------------------ depth 1 = one-step HMC

@pytest.mark.parametrize("kind", ["std", "dense"])
def test_depth_one_is_single_step_hmc_with_random_direction(kind):
    """With max_tree_depth = 1 a NUTS iteration is: draw momentum, one leapfrog step in a random
    direction, Metropolis accept with probability min(1, exp(-dH)).  Re-derived here in numpy."""
    d, eps, seed, n_chains, n_iters = 3, 0.9, 77, 5, 40
    P = np.eye(d) if kind == "std" else W.random_spd_precision(d, 4)
    t = R.Target(R.STD_NORMAL, d) if kind == "std" else R.Target(R.GAUSS_DENSE, d, precision=P)
    st, dep, nl = R.sample(t, n_chains, n_iters, eps, 1, seed)
    assert (dep == 1).all() and (nl == 1).all()
    n_rejected = 0
    for c in range(n_chains):
        x = py_normals(seed, R.TAG_INIT, 0, c, d)
        for it in range(n_iters):
            r = py_normals(seed, R.TAG_MOMENTUM, it, c, d)
            v = 1.0 if (int(R.draw(seed, 0, R.TAG_DIRECTION, 0, it, c)[0]) >> 31) else -1.0
            h = v * eps
            rh = r - 0.5 * h * (P @ x)
            x1 = x + h * rh
            r1 = rh - 0.5 * h * (P @ x1)
            dH = (0.5 * x1 @ P @ x1 + 0.5 * r1 @ r1) - (0.5 * x @ P @ x + 0.5 * r @ r)
            u = float(py_u(seed, 0, R.TAG_TOP, 0, it, c))
            if dH <= 1000 and math.log(u) < -dH:
                x = x1
            else:
                n_rejected += 1
            assert np.allclose(st[it, c], x, rtol=1e-12, atol=1e-13)
    assert n_rejected > 0   # the accept test was exercised both ways


# ------------------------------------------------------------------ exact-arithmetic replay

def exact_iteration(theta, r0, eps, max_depth, seed, it, chain, k=1):
    """One NUTS iteration on the standard normal in exact rational arithmetic (the leapfrog map is
    rational there), weights in 60-digit decimals.  Written over *leaf index ranges*, not as the
    oracle's summary-passing recursion.  A leaf is the k-fold leapfrog map; draws inside a doubling
    are keyed by the leapfrog-step count at the merge.  Returns (depth, n_leapfrog, selected position)."""
    getcontext().prec = 60
    d = len(theta)

    def step(q, p, h):
        ph = [p[i] - h / 2 * q[i] for i in range(d)]
        q1 = [q[i] + h * ph[i] for i in range(d)]
        p1 = [ph[i] - h / 2 * q1[i] for i in range(d)]
        return q1, p1

    def energy(q, p):
        return sum(x * x for x in q) / 2 + sum(x * x for x in p) / 2

    def weight(q, p):
        dH = energy(q, p) - H0
        if dH > 1000:
            return None
        return (Decimal(-dH.numerator) / Decimal(dH.denominator)).exp()

    def no_uturn(lo, hi):       # lo, hi: (q, p) of the backward-most / forward-most points in time
        span = [hi[0][i] - lo[0][i] for i in range(d)]
        return sum(span[i] * lo[1][i] for i in range(d)) >= 0 and sum(span[i] * hi[1][i] for i in range(d)) >= 0

    H0 = energy(theta, r0)
    minus = plus = (theta, r0)
    chosen, W_tree = theta, Decimal(1)
    n_leap = 0
    for j in range(max_depth):
        v = 1 if (int(R.draw(seed, j, R.TAG_DIRECTION, 0, it, chain)[0]) >> 31) else -1
        leaves = []             # generated lazily, in integration order
        start = plus if v > 0 else minus
        base = n_leap

        def leaf(i):
            while len(leaves) <= i:
                q, p = leaves[-1] if leaves else start
                for _ in range(k):
                    q, p = step(q, p, Fraction(v) * eps)
                leaves.append((q, p))
            return leaves[i]

        def subtree(lo, hi):    # -> (valid, total weight, index of selected leaf)
            if hi - lo == 1:
                w = weight(*leaf(lo))
                return (w is not None), (w if w is not None else Decimal(0)), lo
            mid = (lo + hi) // 2
            okL, wL, pL = subtree(lo, mid)
            if not okL:
                return False, wL, pL
            okR, wR, pR = subtree(mid, hi)
            if not okR:
                return False, wL + wR, pL
            level = (hi - lo).bit_length() - 1
            u = py_u(seed, base + k * hi, R.TAG_SUBTREE, level, it, chain)
            pick = pR if Decimal(u.numerator) / Decimal(u.denominator) * (wL + wR) < wR else pL
            a, b = leaf(lo), leaf(hi - 1)
            ok = no_uturn(a, b) if v > 0 else no_uturn(b, a)
            return ok, wL + wR, pick

        ok, w_new, pick = subtree(0, 2**j)
        n_leap = base + k * len(leaves)
        if v > 0:
            plus = leaves[-1]
        else:
            minus = leaves[-1]
        if ok:
            u = py_u(seed, j, R.TAG_TOP, 0, it, chain)
            if Decimal(u.numerator) / Decimal(u.denominator) * W_tree < w_new:
                chosen = leaves[pick][0]
        W_tree += w_new
        if not (ok and no_uturn(minus, plus)):
            return j + 1, n_leap, chosen
    return max_depth, n_leap, chosen


def test_integer_outputs_match_exact_rational_replay_on_config_1():
    """Tree depths and leapfrog counts of configuration 1 recomputed without floating point."""
    w = W.make(1)
    st, dep, nl, margin = R.sample(target_of(w), w.n_chains, w.n_iters, w.step_size, w.max_tree_depth, w.seed,
                                   want_margin=True)
    assert margin.min() > 1e-9   # no decision sits within rounding error of its threshold
    eps = Fraction(w.step_size)
    for c in range(w.n_chains):
        x = py_normals(w.seed, R.TAG_INIT, 0, c, w.dim)
        for it in range(w.n_iters):
            r0 = py_normals(w.seed, R.TAG_MOMENTUM, it, c, w.dim)
            depth, n_leap, chosen = exact_iteration([Fraction(v) for v in x], [Fraction(v) for v in r0], eps,
                                                    w.max_tree_depth, w.seed, it, c)
            assert depth == dep[it, c] and n_leap == nl[it, c], (c, it)
            assert np.allclose([float(v) for v in chosen], st[it, c], rtol=1e-12, atol=1e-13), (c, it)
            x = st[it, c]        # restart from the oracle's own (rounded) state: errors do not build up
    assert dep.min() >= 1 and dep.max() <= w.max_tree_depth and len(np.unique(dep)) >= 3


def test_exact_replay_with_early_exits_and_divergences():
    """Same replay at a step size large enough that subtrees stop early (U-turns inside the new
    half and energy errors above the threshold both occur)."""
    seed, eps, max_depth, d = 5, 1.75, 5, 2
    t = R.Target(R.STD_NORMAL, d)
    rng = np.random.default_rng(0)
    init = rng.standard_normal((6, d)) * np.array([1.0, 40.0])
    st, dep, nl, margin = R.sample(t, 6, 30, eps, max_depth, seed, init_states=init, want_margin=True)
    assert margin.min() > 1e-9
    partial = 0
    for c in range(6):
        x = init[c]
        for it in range(30):
            r0 = py_normals(seed, R.TAG_MOMENTUM, it, c, d)
            depth, n_leap, chosen = exact_iteration([Fraction(v) for v in x], [Fraction(v) for v in r0],
                                                    Fraction(eps), max_depth, seed, it, c)
            assert depth == dep[it, c] and n_leap == nl[it, c], (c, it)
            assert np.allclose([float(v) for v in chosen], st[it, c], rtol=1e-12, atol=1e-12), (c, it)
            partial += n_leap != 2**depth - 1
            x = st[it, c]
    assert partial > 5


# ------------------------------------------------------------------ several leapfrog steps per leaf

@pytest.mark.parametrize("k,eps,scale", [(2, 0.45, 1.0), (4, 0.11, 1.0), (3, 0.3, 1.0), (3, 1.75, 40.0)])
def test_exact_replay_with_several_steps_per_leaf(k, eps, scale):
    """Section 4.1: a leaf may be a fixed number of leapfrog steps.  Replayed without floating point,
    at step sizes with full trees, early exits and (third case) divergent leaves."""
    seed, max_depth, d, n_chains, n_iters = 11, 5, 2, 4, 25
    t = R.Target(R.STD_NORMAL, d)
    init = np.random.default_rng(k).standard_normal((n_chains, d)) * np.array([1.0, scale])
    st, dep, nl, margin = R.sample(t, n_chains, n_iters, eps, max_depth, seed, init_states=init, want_margin=True,
                                   leaf_steps=k)
    assert margin.min() > 1e-9
    assert (nl % k == 0).all()
    for c in range(n_chains):
        x = init[c]
        for it in range(n_iters):
            r0 = py_normals(seed, R.TAG_MOMENTUM, it, c, d)
            depth, n_leap, chosen = exact_iteration([Fraction(v) for v in x], [Fraction(v) for v in r0],
                                                    Fraction(eps), max_depth, seed, it, c, k=k)
            assert depth == dep[it, c] and n_leap == nl[it, c], (c, it)
            assert np.allclose([float(v) for v in chosen], st[it, c], rtol=1e-12, atol=1e-12), (c, it)
            x = st[it, c]
    leaves = nl // k
    if scale == 1.0:
        assert len(np.unique(dep)) >= 3
    else:
        assert (leaves != 2**dep - 1).sum() > 5      # trees cut short by divergent leaves / inner U-turns


def test_one_step_per_leaf_is_the_default_and_leaf_count_bounds_hold():
    w = W.make(3, n_chains=6, n_iters=10)
    t = target_of(w)
    a = R.sample(t, 6, 10, w.step_size, w.max_tree_depth, w.seed)
    b = R.sample(t, 6, 10, w.step_size, w.max_tree_depth, w.seed, leaf_steps=1)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    for k in (2, 4):
        st, dep, nl = R.sample(t, 6, 10, w.step_size / k, w.max_tree_depth, w.seed, leaf_steps=k)
        leaves = nl // k
        assert (nl % k == 0).all() and (leaves >= 2 ** (dep - 1)).all() and (leaves <= 2**dep - 1).all()
        assert not np.array_equal(st, a[0])
    for bad in (0, -1, 65):
        with pytest.raises(ValueError):
            R.sample(t, 2, 2, 0.1, 3, 1, leaf_steps=bad)


def test_depth_one_with_k_steps_is_k_step_hmc():
    """max_tree_depth = 1 and k steps per leaf is plain HMC with k leapfrog steps (numpy re-derivation)."""
    d, eps, seed, k = 3, 0.5, 21, 3
    P = W.random_spd_precision(d, 4)
    t = R.Target(R.GAUSS_DENSE, d, precision=P)
    st, dep, nl = R.sample(t, 4, 30, eps, 1, seed, leaf_steps=k)
    assert (nl == k).all()
    rejected = 0
    for c in range(4):
        x = py_normals(seed, R.TAG_INIT, 0, c, d)
        for it in range(30):
            r = py_normals(seed, R.TAG_MOMENTUM, it, c, d)
            h = eps * (1.0 if (int(R.draw(seed, 0, R.TAG_DIRECTION, 0, it, c)[0]) >> 31) else -1.0)
            q, p = x.copy(), r.copy()
            for _ in range(k):
                p = p - 0.5 * h * (P @ q)
                q = q + h * p
                p = p - 0.5 * h * (P @ q)
            dH = (0.5 * q @ P @ q + 0.5 * p @ p) - (0.5 * x @ P @ x + 0.5 * r @ r)
            if dH <= 1000 and math.log(float(py_u(seed, 0, R.TAG_TOP, 0, it, c))) < -dH:
                x = q
            else:
                rejected += 1
            assert np.allclose(st[it, c], x, rtol=1e-12, atol=1e-13)
    assert rejected > 0


def test_one_dimensional_normal_is_stationary_with_three_steps_per_leaf():
    n = 100000
    x0 = np.random.default_rng(5).standard_normal((n, 1))
    st, dep, nl = R.sample(R.Target(R.STD_NORMAL, 1), n, 2, 0.5, 4, 99, init_states=x0, n_threads=8, leaf_steps=3)
    x = st[1, :, 0]
    assert stats.kstest(x, "norm").pvalue > 1e-3
    assert abs(x.var() - 1) < 4.5 * math.sqrt(2 / n)
    assert abs(np.mean(x**4) - 3) < 4.5 * math.sqrt(96 / n)


# ------------------------------------------------------------------ slice-sampling form (the published algorithm)

def exact_slice_iteration(theta, r0, eps, max_depth, seed, it, chain, k=1):
    """One iteration of slice-sampling NUTS (Hoffman & Gelman, Algorithm 3) on the standard normal in
    exact rational arithmetic, written over leaf index ranges with candidate *lists* instead of the
    oracle's counts: a subtree returns the leaves that lie under the slice, and selection picks
    among them through the same uniforms.  Returns (depth, n_leapfrog, selected position)."""
    getcontext().prec = 60
    d = len(theta)

    def step(q, p, h):
        ph = [p[i] - h / 2 * q[i] for i in range(d)]
        q1 = [q[i] + h * ph[i] for i in range(d)]
        return q1, [ph[i] - h / 2 * q1[i] for i in range(d)]

    def energy(q, p):
        return sum(x * x for x in q) / 2 + sum(x * x for x in p) / 2

    def dec(fr):
        return Decimal(fr.numerator) / Decimal(fr.denominator)

    H0 = energy(theta, r0)
    u_slice = dec(py_u(seed, 0, R.TAG_SLICE, 0, it, chain))     # slice height = u_slice * exp(-H0)

    def under_slice(q, p):      # (candidate, still valid)
        dH = energy(q, p) - H0
        density = (-dec(dH)).exp() if dH < 5000 else Decimal(0)
        return u_slice <= density, (dH < 5000 and u_slice < density * Decimal(1000).exp())

    def no_uturn(lo, hi):
        span = [hi[0][i] - lo[0][i] for i in range(d)]
        return sum(span[i] * lo[1][i] for i in range(d)) >= 0 and sum(span[i] * hi[1][i] for i in range(d)) >= 0

    minus = plus = (theta, r0)
    chosen, n_tree, n_leap = theta, 1, 0
    for j in range(max_depth):
        v = 1 if (int(R.draw(seed, j, R.TAG_DIRECTION, 0, it, chain)[0]) >> 31) else -1
        leaves, start, base = [], (plus if v > 0 else minus), n_leap

        def leaf(i):
            while len(leaves) <= i:
                q, p = leaves[-1] if leaves else start
                for _ in range(k):
                    q, p = step(q, p, Fraction(v) * eps)
                leaves.append((q, p))
            return leaves[i]

        def subtree(lo, hi):    # -> (valid, number of candidates, index of the selected leaf)
            if hi - lo == 1:
                cand, valid = under_slice(*leaf(lo))
                return valid, int(cand), lo
            mid = (lo + hi) // 2
            okL, nL, pL = subtree(lo, mid)
            if not okL:
                return False, nL, pL
            okR, nR, pR = subtree(mid, hi)
            level = (hi - lo).bit_length() - 1
            u = py_u(seed, base + k * hi, R.TAG_SUBTREE, level, it, chain)
            pick = pR if u * (nL + nR) < nR else pL
            if not okR:
                return False, nL + nR, pick
            a, b = leaf(lo), leaf(hi - 1)
            return (no_uturn(a, b) if v > 0 else no_uturn(b, a)), nL + nR, pick

        ok, n_new, pick = subtree(0, 2**j)
        n_leap = base + k * len(leaves)
        if v > 0:
            plus = leaves[-1]
        else:
            minus = leaves[-1]
        if ok and py_u(seed, j, R.TAG_TOP, 0, it, chain) * n_tree < n_new:
            chosen = leaves[pick][0]
        n_tree += n_new
        if not (ok and no_uturn(minus, plus)):
            return j + 1, n_leap, chosen
    return max_depth, n_leap, chosen


@pytest.mark.parametrize("k,eps,scale,max_depth", [(1, 0.5, 1.0, 6), (1, 1.75, 40.0, 5), (3, 0.3, 1.0, 5), (3, 1.75, 40.0, 5)])
def test_slice_sampler_integer_outputs_match_exact_rational_replay(k, eps, scale, max_depth):
    seed, d, n_chains, n_iters = 23, 2, 5, 30
    t = R.Target(R.STD_NORMAL, d)
    init = np.random.default_rng(7 + k).standard_normal((n_chains, d)) * np.array([1.0, scale])
    st, dep, nl, margin = R.sample(t, n_chains, n_iters, eps, max_depth, seed, init_states=init, want_margin=True,
                                   leaf_steps=k, sampler=R.SLICE)
    assert margin.min() > 1e-9
    moved = 0
    for c in range(n_chains):
        x = init[c]
        for it in range(n_iters):
            r0 = py_normals(seed, R.TAG_MOMENTUM, it, c, d)
            depth, n_leap, chosen = exact_slice_iteration([Fraction(v) for v in x], [Fraction(v) for v in r0],
                                                          Fraction(eps), max_depth, seed, it, c, k=k)
            assert depth == dep[it, c] and n_leap == nl[it, c], (c, it)
            assert np.allclose([float(v) for v in chosen], st[it, c], rtol=1e-12, atol=1e-12), (c, it)
            moved += not np.array_equal(st[it, c], x)
            x = st[it, c]
    assert moved > n_chains * n_iters // 3
    leaves = nl // k
    if scale == 1.0:
        assert len(np.unique(dep)) >= 3
    else:
        assert (leaves != 2**dep - 1).sum() > 5


def test_slice_sampler_at_depth_one_is_metropolis_with_the_slice_uniform():
    """With one doubling the only candidate besides the start is the single leaf: it is under the slice
    iff u_slice <= exp(-dH), and it is then always taken (1 candidate against 1)."""
    d, eps, seed = 3, 0.9, 5
    P = W.random_spd_precision(d, 4)
    st, dep, nl = R.sample(R.Target(R.GAUSS_DENSE, d, precision=P), 5, 40, eps, 1, seed, sampler=R.SLICE)
    assert (dep == 1).all() and (nl == 1).all()
    rejected = 0
    for c in range(5):
        x = py_normals(seed, R.TAG_INIT, 0, c, d)
        for it in range(40):
            r = py_normals(seed, R.TAG_MOMENTUM, it, c, d)
            h = eps * (1.0 if (int(R.draw(seed, 0, R.TAG_DIRECTION, 0, it, c)[0]) >> 31) else -1.0)
            rh = r - 0.5 * h * (P @ x)
            x1 = x + h * rh
            r1 = rh - 0.5 * h * (P @ x1)
            dH = (0.5 * x1 @ P @ x1 + 0.5 * r1 @ r1) - (0.5 * x @ P @ x + 0.5 * r @ r)
            if math.log(float(py_u(seed, 0, R.TAG_SLICE, 0, it, c))) <= -dH:
                x = x1
            else:
                rejected += 1
            assert np.allclose(st[it, c], x, rtol=1e-12, atol=1e-13)
    assert rejected > 0


@pytest.mark.parametrize("eps,max_depth,k", [(0.3, 5, 1), (0.9, 4, 1), (1.6, 3, 1), (0.4, 4, 2)])
def test_slice_sampler_leaves_the_normal_invariant(eps, max_depth, k):
    n = 100000
    x0 = np.random.default_rng(321).standard_normal((n, 1))
    st, dep, nl = R.sample(R.Target(R.STD_NORMAL, 1), n, 3, eps, max_depth, 2025, init_states=x0, n_threads=8,
                           leaf_steps=k, sampler=R.SLICE)
    for it in (0, 2):
        x = st[it, :, 0]
        assert stats.kstest(x, "norm").pvalue > 1e-3
        assert abs(x.mean()) < 4.5 / math.sqrt(n)
        assert abs(x.var() - 1) < 4.5 * math.sqrt(2 / n)
        assert abs(np.mean(x**4) - 3) < 4.5 * math.sqrt(96 / n)
    assert np.abs(st[0, :, 0] - x0[:, 0]).mean() > 0.1


def test_slice_sampler_recovers_a_correlated_gaussian_and_differs_from_multinomial():
    d = 4
    P = W.ar1_precision(d, 0.9)
    t = R.Target(R.GAUSS_DENSE, d, precision=P)
    st, dep, nl = R.sample(t, 256, 400, 0.25, 7, 77, n_threads=8, sampler=R.SLICE)
    x = st[100:].reshape(-1, d)
    cov = np.linalg.inv(P)
    assert np.abs(x.mean(axis=0)).max() < 0.08
    assert np.abs(np.cov(x.T) - cov).max() < 0.12
    assert (dep >= 1).all() and (nl >= 2 ** (dep - 1)).all() and (nl <= 2**dep - 1).all()
    other = R.sample(t, 256, 5, 0.25, 7, 77, n_threads=8)
    assert not np.array_equal(other[0], st[:5])
    with pytest.raises(ValueError):
        R.sample(t, 2, 2, 0.1, 3, 1, sampler=2)


# ------------------------------------------------------------------ structure, independence

@pytest.mark.parametrize("cfg,n_chains,n_iters", [(1, 4, 100), (2, 6, 15), (3, 6, 30), (5, 3, 4)])
def test_structural_invariants(cfg, n_chains, n_iters):
    w = W.make(cfg, n_chains=n_chains, n_iters=n_iters)
    st, dep, nl = R.sample(target_of(w), n_chains, n_iters, w.step_size, w.max_tree_depth, w.seed, n_threads=4)
    assert np.isfinite(st).all()
    assert (dep >= 1).all() and (dep <= w.max_tree_depth).all()
    assert (nl >= 2 ** (dep - 1)).all() and (nl <= 2**dep - 1).all()


def test_chains_do_not_depend_on_their_companions_or_on_threads():
    """Section 2 of the paper: every batch member sees the execution it would see alone."""
    w = W.make(3, n_chains=12, n_iters=12)
    t = target_of(w)
    args = (w.step_size, w.max_tree_depth, w.seed)
    full = R.sample(t, 12, 12, *args, n_threads=1)
    again = R.sample(t, 12, 12, *args, n_threads=5)
    ids = np.array([7, 2, 11])
    sub = R.sample(t, 3, 12, *args, chain_ids=ids)
    for a, b, s in zip(full, again, sub):
        assert np.array_equal(a, b)
        assert np.array_equal(a[:, ids], s)
    other = R.sample(t, 12, 12, w.step_size, w.max_tree_depth, w.seed + 1)
    assert not np.array_equal(full[0], other[0])


def test_initial_states_come_from_the_init_draws():
    w = W.make(1)
    t = target_of(w)
    x0 = np.stack([py_normals(w.seed, R.TAG_INIT, 0, c, w.dim) for c in range(4)])
    a = R.sample(t, 4, 10, w.step_size, w.max_tree_depth, w.seed)
    b = R.sample(t, 4, 10, w.step_size, w.max_tree_depth, w.seed, init_states=x0)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    # odd dimension: the second normal of the last block is dropped
    t3 = R.Target(R.STD_NORMAL, 3)
    x0 = np.stack([py_normals(9, R.TAG_INIT, 0, c, 3) for c in range(2)])
    a = R.sample(t3, 2, 5, 0.4, 4, 9)
    b = R.sample(t3, 2, 5, 0.4, 4, 9, init_states=x0)
    assert np.array_equal(a[0], b[0])


def test_f32_oracle_tracks_f64_on_a_short_run():
    w = W.make(2, n_chains=6, n_iters=3)
    a = R.sample(target_of(w, np.float32), 6, 3, w.step_size, w.max_tree_depth, w.seed)
    b = R.sample(target_of(w, np.float64), 6, 3, w.step_size, w.max_tree_depth, w.seed)
    assert a[0].dtype == np.float32
    assert np.array_equal(a[1][0], b[1][0]) and np.array_equal(a[2][0], b[2][0])
    assert np.allclose(a[0][0], b[0][0], atol=1e-4)


def test_argument_checks():
    t = R.Target(R.STD_NORMAL, 2)
    for bad in [dict(n_chains=0), dict(n_iters=0), dict(step_size=0.0), dict(step_size=float("nan")),
                dict(max_tree_depth=0), dict(max_tree_depth=21)]:
        kw = dict(n_chains=2, n_iters=2, step_size=0.1, max_tree_depth=3, seed=1)
        kw.update(bad)
        with pytest.raises(ValueError):
            R.sample(t, **kw)


# ------------------------------------------------------------------ the sampler leaves its target invariant

@pytest.mark.parametrize("eps,max_depth", [(0.3, 5), (0.9, 4), (1.6, 3)])
def test_one_dimensional_normal_is_stationary(eps, max_depth):
    """Chains started from exact N(0,1) draws must still be N(0,1) after 1 and 3 iterations, also at
    step sizes where leaves carry very unequal weights (this is what fixes the selection rules)."""
    n = 100000
    rng = np.random.default_rng(123)
    x0 = rng.standard_normal((n, 1))
    t = R.Target(R.STD_NORMAL, 1)
    st, dep, nl = R.sample(t, n, 3, eps, max_depth, 2024, init_states=x0, n_threads=8)
    for it in (0, 2):
        x = st[it, :, 0]
        assert stats.kstest(x, "norm").pvalue > 1e-3
        assert abs(x.mean()) < 4.5 / math.sqrt(n)
        assert abs(x.var() - 1) < 4.5 * math.sqrt(2 / n)
        assert abs(np.mean(x**4) - 3) < 4.5 * math.sqrt(96 / n)
    assert np.abs(st[0, :, 0] - x0[:, 0]).mean() > 0.1     # and it does move


def test_long_run_histogram_of_a_single_chain_family():
    t = R.Target(R.STD_NORMAL, 1)
    st, _, _ = R.sample(t, 64, 4000, 0.7, 6, 31, n_threads=8)
    x = st[200:, :, 0].ravel()
    edges = np.array([-np.inf, -2, -1, -0.5, 0, 0.5, 1, 2, np.inf])
    freq = np.histogram(x, bins=edges)[0] / x.size
    want = np.diff(stats.norm.cdf(edges))
    assert np.abs(freq - want).max() < 0.004


def test_gaussian_targets_recover_mean_and_covariance():
    d, n_chains, n_iters, warm = 8, 256, 400, 100
    P = W.ar1_precision(d, 0.9)
    S = np.linalg.inv(P)
    t = R.Target(R.GAUSS_DENSE, d, precision=P)
    st, dep, nl = R.sample(t, n_chains, n_iters, 0.25, 8, 11, n_threads=8)
    x = st[warm:]
    per_chain_mean = x.mean(axis=0)                       # [chains, d]
    mcse = per_chain_mean.std(axis=0, ddof=1) / math.sqrt(n_chains)
    assert (np.abs(per_chain_mean.mean(axis=0)) < 4.5 * mcse).all()
    per_chain_cov = np.einsum("tci,tcj->cij", x, x) / x.shape[0]
    cov = per_chain_cov.mean(axis=0)
    cov_se = per_chain_cov.std(axis=0, ddof=1) / math.sqrt(n_chains)
    assert (np.abs(cov - S) < 4.5 * cov_se).all()
    assert np.abs(cov - S).max() < 0.1
    # diagonal target with very different scales
    sig = np.array([0.1, 1.0, 7.0])
    td = R.Target(R.GAUSS_DIAG, 3, scales=sig)
    st, _, _ = R.sample(td, 256, 400, 0.15, 8, 12, n_threads=8)
    v = (st[100:] ** 2).mean(axis=0)
    se = v.std(axis=0, ddof=1) / math.sqrt(256)
    assert (np.abs(v.mean(axis=0) - sig**2) < 4.5 * se).all()


@pytest.mark.parametrize("dim", [1, 2])
def test_tiny_logistic_regression_against_grid_quadrature(dim):
    rng = np.random.default_rng(77 + dim)
    X = rng.standard_normal((5, dim)); X[:, -1] = 1.0
    y = np.array([1.0, 0.0, 1.0, 1.0, 0.0])
    t = R.Target(R.LOGREG, dim, X=X, y=y, prior_scale=1.5)
    # brute force: posterior moments on a grid
    g = np.linspace(-9, 9, 721)
    if dim == 1:
        th = g[:, None]
    else:
        th = np.stack(np.meshgrid(g, g, indexing="ij"), axis=-1).reshape(-1, 2)
    z = th @ X.T
    logpost = (y * z - np.logaddexp(0, z)).sum(axis=1) - 0.5 * (th**2).sum(axis=1) / 1.5**2
    wts = np.exp(logpost - logpost.max()); wts /= wts.sum()
    mean = wts @ th
    second = wts @ th**2
    n_chains, n_iters, warm = 512, 300, 50
    st, _, _ = R.sample(t, n_chains, n_iters, 0.5, 6, 5, n_threads=8)
    x = st[warm:]
    m_c, s_c = x.mean(axis=0), (x**2).mean(axis=0)
    assert (np.abs(m_c.mean(axis=0) - mean) < 4.5 * m_c.std(axis=0, ddof=1) / math.sqrt(n_chains)).all()
    assert (np.abs(s_c.mean(axis=0) - second) < 4.5 * s_c.std(axis=0, ddof=1) / math.sqrt(n_chains)).all()
