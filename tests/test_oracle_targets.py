"""Pins for the oracle's target log-densities and gradients, the leapfrog integrator and the U-turn test."""
import numpy as np
import pytest
from scipy import special, stats

from oracle import nuts_ref as R
from paper_1910_11141_amd import workloads as W


def targets_f64():
    rng = np.random.default_rng(42)
    lr = W.small_logreg(40, 5, seed=9)
    return {
        "std": R.Target(R.STD_NORMAL, 7),
        "dense": R.Target(R.GAUSS_DENSE, 6, precision=W.random_spd_precision(6, 1)),
        "ar1": R.Target(R.GAUSS_DENSE, 9, precision=W.ar1_precision(9, 0.9)),
        "diag": R.Target(R.GAUSS_DIAG, 8, scales=10.0 ** rng.uniform(-1, 1, 8)),
        "logreg": R.Target(R.LOGREG, 5, X=lr.X, y=lr.y, prior_scale=1.0),
        "logreg_prior2": R.Target(R.LOGREG, 5, X=lr.X, y=lr.y, prior_scale=2.5),
    }


@pytest.mark.parametrize("name", list(targets_f64()))
def test_gradient_matches_central_differences(name):
    t = targets_f64()[name]
    rng = np.random.default_rng(0)
    for _ in range(5):
        x = rng.standard_normal(t.dim)
        _, g = R.logp_grad(t, x)
        h = 1e-6
        fd = np.empty(t.dim)
        for i in range(t.dim):
            e = np.zeros(t.dim); e[i] = h
            fd[i] = (R.logp_grad(t, x + e)[0] - R.logp_grad(t, x - e)[0]) / (2 * h)
        assert np.allclose(g, fd, rtol=1e-7, atol=1e-7 * max(1.0, np.abs(g).max()))


def test_gaussian_logp_against_scipy_densities():
    ts = targets_f64()
    rng = np.random.default_rng(1)
    x, x2 = rng.standard_normal(7), rng.standard_normal(7)
    assert R.logp_grad(ts["std"], x)[0] == pytest.approx(stats.norm.logpdf(x).sum() + 3.5 * np.log(2 * np.pi), rel=1e-14)
    for name in ("dense", "ar1"):
        t = ts[name]
        mvn = stats.multivariate_normal(mean=np.zeros(t.dim), cov=np.linalg.inv(t.precision))
        a, b = rng.standard_normal(t.dim), rng.standard_normal(t.dim)
        assert R.logp_grad(t, a)[0] - R.logp_grad(t, b)[0] == pytest.approx(mvn.logpdf(a) - mvn.logpdf(b), rel=1e-10)
        assert np.allclose(R.logp_grad(t, a)[1], -t.precision @ a, rtol=1e-13)
    t = ts["diag"]
    a, b = rng.standard_normal(8), rng.standard_normal(8)
    want = stats.norm.logpdf(a, scale=t.scales).sum() - stats.norm.logpdf(b, scale=t.scales).sum()
    assert R.logp_grad(t, a)[0] - R.logp_grad(t, b)[0] == pytest.approx(want, rel=1e-11)
    assert np.allclose(R.logp_grad(t, a)[1], -a / t.scales**2, rtol=1e-14)


def test_ar1_precision_is_the_inverse_of_the_stated_covariance():
    P = W.ar1_precision(100, 0.9)
    i = np.arange(100)
    S = 0.9 ** np.abs(i[:, None] - i[None, :])
    assert np.allclose(P @ S, np.eye(100), atol=1e-10)


def test_logreg_logp_against_scipy_bernoulli_and_normal():
    for name, s in (("logreg", 1.0), ("logreg_prior2", 2.5)):
        t = targets_f64()[name]
        rng = np.random.default_rng(2)
        th = rng.standard_normal(t.dim)
        z = t.X @ th
        want = stats.bernoulli.logpmf(t.y.astype(int), special.expit(z)).sum() \
            + stats.norm.logpdf(th, scale=s).sum() + t.dim * (0.5 * np.log(2 * np.pi) + np.log(s))
        lp, g = R.logp_grad(t, th)
        assert lp == pytest.approx(want, rel=1e-12)
        assert np.allclose(g, t.X.T @ (t.y - special.expit(z)) - th / s**2, rtol=1e-12, atol=1e-13)


def test_logreg_is_stable_for_huge_logits():
    X = np.array([[1000.0], [-1000.0], [40.0], [-40.0], [0.0]])
    y = np.array([1.0, 1.0, 0.0, 0.0, 1.0])
    t = R.Target(R.LOGREG, 1, X=X, y=y)
    lp, g = R.logp_grad(t, np.array([1.0]))
    # terms: y z - softplus(z): 0, -1000, -40-log1p(e^-40), -log1p(e^-40), -log 2 ; prior -1/2
    want = 0.0 - 1000.0 - 40.0 - 2 * np.log1p(np.exp(-40.0)) - np.log(2.0) - 0.5
    assert np.isfinite(lp) and lp == pytest.approx(want, rel=1e-15)
    resid = np.array([0.0, 1.0, -1.0, -special.expit(-40.0), 0.5])
    assert g[0] == pytest.approx(float(X[:, 0] @ resid) - 1.0, rel=1e-13)


def test_diag_dense_and_std_kinds_agree_bit_for_bit():
    rng = np.random.default_rng(3)
    d = 11
    sig = 10.0 ** rng.uniform(-1, 1, d)
    P = np.diag(1.0 / (sig * sig))
    td, tD = R.Target(R.GAUSS_DIAG, d, scales=sig), R.Target(R.GAUSS_DENSE, d, precision=P)
    ts, t1 = R.Target(R.STD_NORMAL, d), R.Target(R.GAUSS_DIAG, d, scales=np.ones(d))
    for _ in range(20):
        x = rng.standard_normal(d) * 3
        (la, ga), (lb, gb) = R.logp_grad(td, x), R.logp_grad(tD, x)
        assert la == lb and np.array_equal(ga, gb)
        (la, ga), (lb, gb) = R.logp_grad(ts, x), R.logp_grad(t1, x)
        assert la == lb and np.array_equal(ga, gb)


def test_f32_targets_track_f64():
    rng = np.random.default_rng(4)
    lr = W.small_logreg(300, 6, seed=10)
    pairs = [
        (R.Target(R.LOGREG, 6, np.float32, X=lr.X, y=lr.y), R.Target(R.LOGREG, 6, np.float64, X=lr.X.astype(np.float32), y=lr.y)),
        (R.Target(R.GAUSS_DENSE, 6, np.float32, precision=W.random_spd_precision(6, 2)),
         R.Target(R.GAUSS_DENSE, 6, np.float64, precision=W.random_spd_precision(6, 2).astype(np.float32))),
    ]
    for t32, t64 in pairs:
        x = rng.standard_normal(6).astype(np.float32)
        l32, g32 = R.logp_grad(t32, x)
        l64, g64 = R.logp_grad(t64, x)
        assert g32.dtype == np.float32
        assert l32 == pytest.approx(l64, rel=1e-14)          # reductions are binary64 in both
        assert np.array_equal(g32, g64.astype(np.float32))   # one rounding at the end


# ----------------------------------------------------------------------------- leapfrog

@pytest.mark.parametrize("name", list(targets_f64()))
def test_leapfrog_is_reversible(name):
    t = targets_f64()[name]
    rng = np.random.default_rng(5)
    eps = 0.05 if name == "diag" else 0.1
    for L in (1, 7, 40):
        x, r = rng.standard_normal(t.dim), rng.standard_normal(t.dim)
        x1, r1, _ = R.leapfrog(t, x, r, eps, L)
        x2, r2, _ = R.leapfrog(t, x1, -r1, eps, L)
        assert np.abs(x2 - x).max() < 1e-12 and np.abs(-r2 - r).max() < 1e-12
        # a backward step is a forward step with the sign of eps flipped
        x3, r3, _ = R.leapfrog(t, x1, r1, -eps, L)
        assert np.abs(x3 - x).max() < 1e-12 and np.abs(r3 - r).max() < 1e-12


def test_std_normal_leapfrog_is_the_closed_form_linear_map():
    t = R.Target(R.STD_NORMAL, 4)
    rng = np.random.default_rng(6)
    for eps in (0.5, -0.5, 0.1, 1.3):
        M = np.array([[1 - eps**2 / 2, eps], [-eps * (1 - eps**2 / 4), 1 - eps**2 / 2]])
        assert np.linalg.det(M) == pytest.approx(1.0, rel=1e-15)
        x, r = rng.standard_normal(4), rng.standard_normal(4)
        for L in (1, 2, 9):
            ML = np.linalg.matrix_power(M, L)
            x1, r1, lp = R.leapfrog(t, x, r, eps, L)
            assert np.allclose(x1, ML[0, 0] * x + ML[0, 1] * r, rtol=1e-13, atol=1e-14)
            assert np.allclose(r1, ML[1, 0] * x + ML[1, 1] * r, rtol=1e-13, atol=1e-14)
            assert lp == pytest.approx(-0.5 * x1 @ x1, rel=1e-14)
            # the modified energy (1 - eps^2/4) x^2 + r^2 is conserved exactly
            q0 = (1 - eps**2 / 4) * x**2 + r**2
            q1 = (1 - eps**2 / 4) * x1**2 + r1**2
            assert np.allclose(q0, q1, rtol=1e-13)


def test_dense_gaussian_leapfrog_is_the_closed_form_linear_map():
    d = 6
    P = W.random_spd_precision(d, 8)
    t = R.Target(R.GAUSS_DENSE, d, precision=P)
    eps = 0.2
    I = np.eye(d)
    A = I - eps**2 / 2 * P
    M = np.block([[A, eps * I], [-eps * P @ (I - eps**2 / 4 * P), A]])
    rng = np.random.default_rng(7)
    x, r = rng.standard_normal(d), rng.standard_normal(d)
    for L in (1, 5):
        out = np.linalg.matrix_power(M, L) @ np.concatenate([x, r])
        x1, r1, _ = R.leapfrog(t, x, r, eps, L)
        assert np.allclose(np.concatenate([x1, r1]), out, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("name", ["std", "dense", "ar1", "diag"])
def test_energy_error_is_second_order(name):
    t = targets_f64()[name]
    rng = np.random.default_rng(8)
    x, r = rng.standard_normal(t.dim), rng.standard_normal(t.dim)
    base = 0.02 if name == "diag" else 0.1

    def max_err(eps):
        n = int(round(2.0 / eps))
        H0 = -R.logp_grad(t, x)[0] + 0.5 * r @ r
        worst = 0.0
        for L in range(1, n + 1, max(1, n // 20)):
            x1, r1, lp = R.leapfrog(t, x, r, eps, L)
            worst = max(worst, abs(-lp + 0.5 * r1 @ r1 - H0))
        return worst
    ratio = max_err(base) / max_err(base / 2)
    assert 3.5 < ratio < 4.5


def test_f32_leapfrog_tracks_f64():
    P = W.random_spd_precision(5, 11)
    t32 = R.Target(R.GAUSS_DENSE, 5, np.float32, precision=P)
    t64 = R.Target(R.GAUSS_DENSE, 5, np.float64, precision=P)
    rng = np.random.default_rng(9)
    x, r = rng.standard_normal(5), rng.standard_normal(5)
    a = R.leapfrog(t32, x, r, 0.1, 20)
    b = R.leapfrog(t64, x, r, 0.1, 20)
    assert a[0].dtype == np.float32
    assert np.allclose(a[0], b[0], atol=2e-5) and np.allclose(a[1], b[1], atol=2e-5)


# ----------------------------------------------------------------------------- U-turn

def test_uturn_rule():
    tm, tp = np.array([0.0, 0.0]), np.array([1.0, 0.0])
    assert R.uturn_ok(tm, [1.0, 0.0], tp, [1.0, 0.0])            # still moving apart
    assert not R.uturn_ok(tm, [1.0, 0.0], tp, [-0.1, 5.0])       # forward end turned back
    assert not R.uturn_ok(tm, [-0.1, 0.0], tp, [1.0, 0.0])       # backward end turned back
    assert R.uturn_ok(tm, [0.0, 3.0], tp, [0.0, -2.0])           # exactly perpendicular: >= 0 continues
    assert R.uturn_ok(tm, [1.0, 0.0], tm, [-1.0, 0.0])           # zero span
    # not symmetric in its two ends: swapping them flips the sign of the span
    assert not R.uturn_ok(tp, [1.0, 0.0], tm, [1.0, 0.0])
    rng = np.random.default_rng(10)
    for _ in range(200):
        a, b, c, d = rng.standard_normal((4, 5))
        want = ((c - a) @ b >= 0) and ((c - a) @ d >= 0)
        assert R.uturn_ok(a, b, c, d) == want
