"""Parity of the HIP path with the CPU oracle, through the C ABI, on a real MI355X.

Bar (from the benchmark definition): tree depths and leapfrog counts bit-exact in binary64 over the
first 50 iterations, states within 1e-10 relative (binary64) or 1e-4 (binary32, short runs).
"""
import json
import os

import numpy as np
import pytest

from oracle import nuts_ref as R
from paper_1910_11141_amd import workloads as W

pytestmark = pytest.mark.gpu

F64_TOL = 1e-10
F32_TOL = 1e-4


def N():
    import paper_1910_11141_amd.binding as B
    return B


def gpu_target(w, dtype=None):
    return N().Target(w.kind, w.dim, dtype or w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y,
                      prior_scale=w.prior_scale)


def ref_target(w, dtype=None):
    return R.Target(w.kind, w.dim, dtype or w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y,
                    prior_scale=w.prior_scale)


def gpu_run(w, variant=0, init=None, first_chain=0, n_chains=None, n_iters=None, tgt=None, leaf_steps=1, schedule=0,
            sampler=0):
    import torch
    B = N()
    tgt = tgt or gpu_target(w)
    nc, ni = n_chains or w.n_chains, n_iters or w.n_iters
    dev_init = None
    if init is not None:
        dev_init = torch.as_tensor(np.ascontiguousarray(init, dtype=w.dtype)).cuda()
    s, d, n = B.nuts_sample(tgt, nc, ni, w.step_size, w.max_tree_depth, w.seed, variant=variant,
                            init_states=dev_init, first_chain=first_chain, leaf_steps=leaf_steps,
                            schedule=schedule, sampler=sampler)
    torch.cuda.synchronize()
    return s.cpu().numpy(), d.cpu().numpy(), n.cpu().numpy(), B.nuts_get_stats(tgt)


def ref_run(w, chain_ids=None, init=None, n_chains=None, n_iters=None, leaf_steps=1, sampler=0):
    nc = len(chain_ids) if chain_ids is not None else (n_chains or w.n_chains)
    return R.sample(ref_target(w), nc, n_iters or w.n_iters, w.step_size, w.max_tree_depth, w.seed,
                    chain_ids=chain_ids, init_states=init, n_threads=8, want_margin=True, leaf_steps=leaf_steps,
                    sampler=sampler)


def state_error(gs, rs):
    """Largest error of any state component relative to that component's own scale: the oracle's largest
    magnitude of the same coordinate over the compared iterations and chains.  (A norm over all coordinates
    would let a coordinate of small scale be wrong by its whole size beside one of large scale.)"""
    if rs.size == 0:
        return 0.0
    scale = np.abs(rs).max(axis=(0, 1))
    scale = np.where(scale > 0, scale, 1.0)
    return float((np.abs(gs - rs) / scale).max())


def report(kind, **fields):
    """Measured agreement figures, one JSON line each, if NUTS_TEST_REPORT names a file (how the figures in the
    design notes were collected)."""
    path = os.environ.get("NUTS_TEST_REPORT")
    if path:
        with open(path, "a") as f:
            f.write(json.dumps(dict(kind=kind, test=os.environ.get("PYTEST_CURRENT_TEST", ""), **fields)) + "\n")


def assert_parity(gpu, ref, tol, cols=None, exact_ints=True, label=""):
    gs, gd, gn = gpu[:3]
    rs, rd, rn, margin = ref
    if cols is not None:
        gs, gd, gn = gs[:, cols], gd[:, cols], gn[:, cols]
    if exact_ints:
        bad = np.argwhere((gd != rd) | (gn != rn))
        assert bad.size == 0, f"{label}: integer outputs differ first at (iter, chain) {bad[0]}, " \
                              f"oracle decision margin there {margin[tuple(bad[0])]:.3e}"
    err = state_error(gs, rs)
    report("f64", label=label, err=err)
    assert err <= tol, f"{label}: states differ by {err:.3e} relative to their coordinate's scale (tolerance {tol})"
    return err


def check_invariants(w, d, n):
    assert (d >= 1).all() and (d <= w.max_tree_depth).all()
    assert (n >= 2 ** (d.astype(np.int64) - 1)).all() and (n <= 2 ** d.astype(np.int64) - 1).all()


# ------------------------------------------------------------------ the five configurations

def test_config1_std_normal_full():
    w = W.make(1)
    g = gpu_run(w)
    assert_parity(g, ref_run(w), F64_TOL, label=w.name)
    assert g[3]["leaf_slots_useful"] == g[2].sum()


def test_config2_dense_gaussian_full_chain_count_first_50_iterations():
    w = W.make(2, n_iters=50)
    g = gpu_run(w)
    check_invariants(w, g[1], g[2])
    ids = np.array([0, 1, 2, 3, 500, 777, 1022, 1023])
    assert_parity(g, ref_run(w, chain_ids=ids), F64_TOL, cols=ids, label=w.name)


def test_config3_logreg_full_chain_count_first_50_iterations_wave_kernel():
    w = W.make(3, n_iters=50)
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_WAVE)
    check_invariants(w, g[1], g[2])
    assert np.isfinite(g[0]).all()
    ids = np.concatenate([np.arange(16), np.random.default_rng(0).choice(4096, 32, replace=False), [4095]])
    assert_parity(g, ref_run(w, chain_ids=ids), F64_TOL, cols=ids, label=w.name)
    st = g[3]
    assert st["leaf_slots_useful"] == g[2].sum() and st["extra_grad_evals"] == w.n_chains


def test_config4_large_logreg_f32_short_wave_kernel():
    w = W.make(4, n_chains=4, n_iters=4)
    g = gpu_run(w, variant=1)
    r = ref_run(w)
    # binary32 run: integer outputs are compared too, but a flipped decision is reported, not fatal
    f32_parity(g, r)


def test_config5_diag_gaussian_f32_short():
    w = W.make(5, n_chains=64, n_iters=20)
    g = gpu_run(w)
    r = ref_run(w)
    check_invariants(w, g[1], g[2])
    f32_parity(g, r)


# ------------------------------------------------------------------ ragged shapes and degenerate cases

@pytest.mark.parametrize("variant", [1, 3])
@pytest.mark.parametrize("dim", [1, 2, 3, 63, 64, 65, 130, 257, 512])
def test_std_normal_ragged_dimensions(dim, variant):
    w = W.Workload(f"std_d{dim}", W.STD_NORMAL, dim, np.dtype(np.float64), 9, 12, 0.35, 7, seed=5)
    g = gpu_run(w, variant=variant)
    assert g[3]["variant"] == variant
    assert_parity(g, ref_run(w), F64_TOL, label=w.name)


@pytest.mark.parametrize("dim", [1, 5, 64, 97])
def test_dense_gaussian_ragged_dimensions(dim):
    w = W.Workload(f"dense_d{dim}", W.GAUSS_DENSE, dim, np.dtype(np.float64), 7, 10, 0.2, 7, seed=6,
                   precision=W.random_spd_precision(dim, 3))
    assert_parity(gpu_run(w), ref_run(w), F64_TOL, label=w.name)


@pytest.mark.parametrize("dim,variant", [(1, 1), (1, 3), (66, 1), (66, 3), (129, 3), (500, 3), (1000, 1)])
def test_diag_gaussian_ragged_dimensions_f64(dim, variant):
    sig = 10.0 ** np.random.default_rng(dim).uniform(-1, 1, dim)
    w = W.Workload(f"diag_d{dim}", W.GAUSS_DIAG, dim, np.dtype(np.float64), 6, 8, 0.05, 8, seed=7, scales=sig)
    g = gpu_run(w, variant=variant)
    assert g[3]["variant"] == variant
    assert_parity(g, ref_run(w), F64_TOL, label=w.name)


@pytest.mark.parametrize("dim", [1, 5, 255, 256, 257, 1000, 1024])
def test_diag_gaussian_f32_register_kernel_is_bit_exact_on_short_runs(dim):
    """binary32 element-wise arithmetic is specified without fused multiply-add, reductions are binary64:
    over a few iterations the register kernel reproduces the oracle's integers exactly."""
    sig = (10.0 ** np.random.default_rng(dim).uniform(-1, 1, dim)).astype(np.float32)
    w = W.Workload(f"diag32_d{dim}", W.GAUSS_DIAG, dim, np.dtype(np.float32), 10, 6, 0.05, 8, seed=17, scales=sig)
    g = gpu_run(w, variant=3)
    r = ref_run(w)
    assert g[3]["variant"] == 3
    assert np.array_equal(g[1], r[1]) and np.array_equal(g[2], r[2])
    assert state_error(g[0], r[0]) <= F32_TOL


@pytest.mark.parametrize("n_data,dim", [(1, 1), (5, 2), (63, 3), (64, 16), (65, 17), (1000, 25), (257, 33), (300, 70)])
def test_logreg_ragged_shapes_wave_kernel(n_data, dim):
    w = W.small_logreg(n_data, dim, seed=100 + n_data)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 10, 12, 0.15 / np.sqrt(max(n_data, 1) / 10), 7
    B = N()
    assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_WAVE), ref_run(w), F64_TOL, label=w.name)


def test_logreg_prior_scale_is_honoured():
    w = W.small_logreg(40, 4, seed=3)
    w.prior_scale = 2.5
    w.n_chains, w.n_iters = 6, 15
    B = N()
    assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_WAVE), ref_run(w), F64_TOL, label="prior 2.5")


@pytest.mark.parametrize("variant", [1, 3])
def test_deep_trees_use_every_frame_level(variant):
    w = W.Workload("deep", W.STD_NORMAL, 2, np.dtype(np.float64), 5, 3, 0.004, 10, seed=8)
    g = gpu_run(w, variant=variant)
    r = ref_run(w)
    assert r[1].max() == 10 and r[2].max() == 1023
    assert_parity(g, r, F64_TOL, label="deep trees")


@pytest.mark.parametrize("variant", [1, 3])
def test_maximum_depth_limit_20_is_accepted(variant):
    w = W.Workload("cap20", W.STD_NORMAL, 3, np.dtype(np.float64), 4, 6, 0.3, 20, seed=9)
    assert_parity(gpu_run(w, variant=variant), ref_run(w), F64_TOL, label="max_tree_depth 20")


def test_depth_one_and_single_chain_single_iteration():
    w = W.Workload("d1", W.STD_NORMAL, 4, np.dtype(np.float64), 1, 1, 0.9, 1, seed=10)
    assert_parity(gpu_run(w), ref_run(w), F64_TOL, label="1x1, depth 1")
    w.n_chains, w.n_iters = 7, 25
    assert_parity(gpu_run(w), ref_run(w), F64_TOL, label="depth 1")


@pytest.mark.parametrize("variant", [1, 3])
def test_divergent_leaves_and_early_exits(variant):
    rng = np.random.default_rng(0)
    init = rng.standard_normal((12, 2)) * np.array([1.0, 40.0])
    w = W.Workload("div", W.STD_NORMAL, 2, np.dtype(np.float64), 12, 30, 1.75, 5, seed=5)
    g = gpu_run(w, init=init, variant=variant)
    r = ref_run(w, init=init)
    assert (r[2] != 2 ** r[1].astype(np.int64) - 1).sum() > 5      # partial trees do occur
    assert_parity(g, r, F64_TOL, label="divergent")


@pytest.mark.parametrize("variant", [1, 3])
def test_non_finite_energy_is_a_divergence_not_a_trap(variant):
    init = np.full((3, 2), 1e200)
    w = W.Workload("inf", W.STD_NORMAL, 2, np.dtype(np.float64), 3, 4, 0.5, 4, seed=2)
    g = gpu_run(w, init=init, variant=variant)
    r = ref_run(w, init=init)
    assert (g[1] == 1).all() and (g[2] == 1).all()
    assert np.array_equal(g[1], r[1]) and np.array_equal(g[2], r[2])
    assert np.array_equal(g[0], r[0])       # every proposal is rejected: the state never moves


def test_tile_kernel_logistic_function_is_accurate_to_rounding():
    import torch
    B = N()
    rng = np.random.default_rng(0)
    z = np.concatenate([rng.normal(scale=s, size=200000) for s in (0.1, 1.0, 5.0, 30.0)] +
                       [np.linspace(-70, 70, 100001), np.arange(0, 38 * 16 + 3) / 16.0,
                        np.nextafter(np.arange(1, 38 * 16 + 3) / 16.0, 0),
                        np.array([0.0, -0.0, 1e-300, 36.99, 37.0, 64.0, 745.0, 1e6, 1e300])])
    from paper_1910_11141_amd import ubench
    v, s = ubench.logistic(torch.as_tensor(z).cuda())
    v, s = v.cpu().numpy(), s.cpu().numpy()
    a = np.abs(z)
    want_v = 0.5 * a + np.log1p(np.exp(-a))
    assert (np.abs(v - want_v) <= 3e-16 * np.maximum(1.0, want_v)).all()
    assert np.abs(s - 0.5 * np.tanh(0.5 * a)).max() < 1e-15
    bad = np.array([np.nan, np.inf, -np.inf])
    v, s = ubench.logistic(torch.as_tensor(bad).cuda())
    assert not np.isfinite(v.cpu().numpy()).any()      # non-finite logits poison the log-density, never a trap
    # the logarithm of the product of sigmas (one per lane and round): products of up to 256 factors in [1/2, 1]
    x = np.concatenate([rng.uniform(0.5, 1.0, 200000), np.exp(-rng.uniform(0, 180, 200000)),
                        0.5 + (np.arange(0, 129) / 256.0), np.nextafter(0.5 + (np.arange(1, 129) / 256.0), 0),
                        2.0 ** -np.arange(0, 300), [1.0, np.nextafter(1.0, 0), 2.0 ** -256 * 1.999]])
    x = x[x <= 1.0]
    got = ubench.log_unit(torch.as_tensor(x).cuda()).cpu().numpy()
    want = np.log(x)
    assert (np.abs(got - want) <= 4.5e-16 * np.maximum(np.abs(want), 0.25)).all()   # 2 ulp; 1e-16 absolute next to x = 1
    assert np.isnan(ubench.log_unit(torch.as_tensor(np.array([np.nan])).cuda()).cpu().numpy()).all()
    # the sine and cosine of the Box-Muller draws: angles 2 pi u on a fine grid, at and next to every quarter turn
    quarter = np.arange(0, 5) * (np.pi / 2)
    phi = np.concatenate([2 * np.pi * rng.uniform(0, 1, 400000), 2 * np.pi * (np.arange(0, 4097) / 4096.0),
                          quarter, np.nextafter(quarter, 7.0)[:-1], np.nextafter(quarter, -1.0)[1:],
                          (np.arange(0, 8) + 0.5) * (np.pi / 4), [2.0 ** -53 * 2 * np.pi, 1e-300]])
    phi = phi[(phi >= 0) & (phi <= 2 * np.pi)]
    sn, cs = ubench.circle_point(torch.as_tensor(phi).cuda())
    # numpy's sin and cos are within an ulp of the true values; absolute next to a zero of the function, where
    # the angle's own rounding (2e-16 of a turn) is all there is
    assert np.abs(sn.cpu().numpy() - np.sin(phi)).max() <= 2.3e-16
    assert np.abs(cs.cpu().numpy() - np.cos(phi)).max() <= 2.3e-16
    # the exponential that makes a leaf's weight from its energy error: everyday errors, the whole range, the edges
    x = np.concatenate([rng.normal(0, 1, 300000), rng.uniform(-745, 700, 300000), np.arange(-1100, 701) * 1.0,
                        (np.arange(-1080, 1010) + 0.5) * np.log(2.0) / 1.0, [0.0, -0.0, 700.0, -745.2, -800.0, -1e300, -np.inf]])
    x = x[x <= 700.0]
    got = ubench.exp_bounded(torch.as_tensor(x).cuda()).cpu().numpy()
    want = np.exp(x)
    normal = want > 2.3e-308
    assert (np.abs(got[normal] - want[normal]) <= 3.4e-16 * want[normal]).all()     # 1.5 ulp
    assert (np.abs(got[~normal] - want[~normal]) <= 1e-323 + 3.4e-16 * want[~normal]).all()   # subnormal results and 0


# ------------------------------------------------------------------ tile kernel (8 chains in lock step, MFMA gradient)

def test_config3_logreg_full_chain_count_first_50_iterations_tile_kernel():
    w = W.make(3, n_iters=50)
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE)
    assert g[3]["variant"] == B.NUTS_VARIANT_TILE
    check_invariants(w, g[1], g[2])
    assert np.isfinite(g[0]).all()
    ids = np.concatenate([np.arange(16), np.random.default_rng(1).choice(4096, 48, replace=False), [4095]])
    assert_parity(g, ref_run(w, chain_ids=ids), F64_TOL, cols=ids, label=w.name)
    st = g[3]
    assert st["leaf_slots_useful"] == g[2].sum() and st["extra_grad_evals"] == w.n_chains
    assert st["leaf_slots_issued"] >= st["leaf_slots_useful"] + st["extra_grad_evals"]
    assert st["occupancy"] > 0.8


def test_auto_variant_picks_the_tile_kernel_for_config3():
    w = W.make(3, n_chains=64, n_iters=5)
    B = N()
    g = gpu_run(w)
    assert g[3]["variant"] == B.NUTS_VARIANT_TILE
    assert_parity(g, ref_run(w), F64_TOL, label="auto")


@pytest.mark.parametrize("n_data,dim", [(1, 1), (5, 2), (63, 3), (64, 16), (65, 17), (1000, 25), (129, 32), (2100, 31)])
def test_logreg_ragged_shapes_tile_kernel(n_data, dim):
    w = W.small_logreg(n_data, dim, seed=100 + n_data)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 21, 12, 0.15 / np.sqrt(max(n_data, 1) / 10), 7
    B = N()
    assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_TILE), ref_run(w), F64_TOL, label=w.name)


def test_tile_kernel_many_rows_folds_the_product_of_sigmas():
    """More than 64 row tiles per wave (8192 rows): the running product of sigmas is folded into a logarithm between
    chunks of tiles; and 40 000 rows, where an unfolded product of up to 5000 factors per lane would underflow."""
    B = N()
    for n_data, n_chains in ((9000, 5), (40000, 3)):
        w = W.small_logreg(n_data, 4, seed=7 + n_data)
        w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = n_chains, 4, 0.15 / np.sqrt(n_data / 10), 5
        g = gpu_run(w, variant=B.NUTS_VARIANT_TILE)
        assert np.isfinite(g[0]).all()
        assert_parity(g, ref_run(w), F64_TOL, label=w.name)


@pytest.mark.parametrize("where,value", [("first", 1.0), ("middle", -2.5), ("none", 0.0), ("two", 3.0), ("zeros", 0.0)])
def test_tile_kernel_constant_column_anywhere_or_absent(where, value):
    """Columns that are the same in every row (the data recipe has one, the intercept): wherever they stand, whatever
    their value, and also when there is none, more than one, or one of zeros (which stays an ordinary column)."""
    w = W.small_logreg(77, 9, seed=31)
    X = w.X.copy()
    rng = np.random.default_rng(5)
    X[:, -1] = rng.standard_normal(77)             # no constant column left
    if where == "first":
        X[:, 0] = value
    elif where == "middle":
        X[:, 4] = value
    elif where == "two":
        X[:, 2] = value
        X[:, 6] = -value
    elif where == "zeros":
        X[:, 3] = 0.0
    w.X = X
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 19, 10, 0.05, 7
    B = N()
    assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_TILE), ref_run(w), F64_TOL, label=f"constant column {where}")


@pytest.mark.parametrize("n_data,dim,col,value", [
    (1, 5, 0, 1.0), (7, 5, 4, 1.0), (16, 5, 2, -2.5), (128, 13, 12, 1.0), (131, 13, 0, 0.5), (300, 17, 16, 1.0),
    (129, 21, 7, 3.0), (2049, 29, 28, 1.0), (1000, 25, 0, 1.0), (40000, 5, 4, 1.0)])
def test_tile_kernel_constant_column_is_the_initial_value_of_the_first_gemm(n_data, dim, col, value):
    """With d = 1 mod 4 a constant column stays out of the first GEMM (one k-step less) and its share of every logit
    is the accumulators' initial value: every such d with both feature-tile counts, the column first, last and in
    between, row counts that fill the last tile, leave it ragged (its filler rows must start from zero, not from the
    column's share), give some waves no tile at all, and need the product of sigmas folded between chunks of tiles."""
    w = W.small_logreg(n_data, dim, seed=500 + n_data + dim)
    X = w.X.copy()
    X[:, -1] = np.random.default_rng(n_data).standard_normal(n_data)   # the recipe's own constant column goes
    X[:, col] = value
    w.X = X
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 19, 8, 0.15 / np.sqrt(max(n_data, 1) / 10), 6
    if n_data == 40000:
        w.n_chains, w.n_iters = 3, 4
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE)
    assert np.isfinite(g[0]).all()
    assert_parity(g, ref_run(w), F64_TOL, label=f"constant column {col} of {dim}, {n_data} rows")
    if n_data in (7, 131):
        assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_TILE, sampler=1, leaf_steps=2), ref_run(w, sampler=1, leaf_steps=2),
                      F64_TOL, label="constant column, slice sampler")


def test_tile_kernel_deep_trees_and_depth_limit():
    w = W.small_logreg(30, 3, seed=4)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 18, 3, 0.002, 10
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE)
    r = ref_run(w)
    assert r[1].max() == 10 and r[2].max() == 1023
    assert_parity(g, r, F64_TOL, label="tile deep")
    w.max_tree_depth = 12
    w.n_iters = 1
    assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_TILE), ref_run(w), F64_TOL, label="tile depth 12")


@pytest.mark.parametrize("dim", [4, 5])   # (5: the constant column is the first GEMM's initial value)
def test_tile_kernel_divergences_and_non_finite_states(dim):
    w = W.small_logreg(50, dim, seed=6)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 20, 20, 0.6, 6
    B = N()
    rng = np.random.default_rng(1)
    init = rng.standard_normal((20, dim)) * 5
    init[3] = 1e200
    init[7] = np.inf
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE, init=init)
    r = ref_run(w, init=init)
    assert (r[2] != 2 ** r[1].astype(np.int64) - 1).sum() > 5
    gs, rs = g[0].copy(), r[0].copy()
    assert np.array_equal(np.isfinite(gs), np.isfinite(rs))
    assert np.array_equal(g[1], r[1]) and np.array_equal(g[2], r[2])
    fin = np.isfinite(rs).all(axis=(0, 2))
    assert fin.sum() == 19 and not fin[7]
    assert state_error(gs[:, fin], rs[:, fin]) < F64_TOL


@pytest.mark.parametrize("scale, eps", [(60.0, 0.6), (300.0, 0.3)])
def test_tile_kernel_energy_far_below_the_start_moves_the_unit_of_the_weights(scale, eps):
    """The tile kernel keeps a trajectory's weights as numbers exp(H0 - H) in a unit that it moves when a leaf's energy
    falls more than 600 below it.  From starting points this far out (the prior term alone is -scale^2 d / 2) leapfrog
    steps of this size land hundreds to tens of thousands below the starting energy in the first trajectories (a plain
    numpy leapfrog of the same set-up shows it for 18 of 20 chains at scale 60 and for all at 300), and others diverge."""
    w = W.small_logreg(50, 4, seed=6)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 20, 10, eps, 6
    B = N()
    init = np.random.default_rng(1).standard_normal((20, 4)) * scale
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE, init=init)
    r = ref_run(w, init=init)
    assert_parity(g, r, F64_TOL, label=f"tile, start at {scale} sigma")
    for steps in (1, 3):
        assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_TILE, init=init, leaf_steps=steps, sampler=1),
                      ref_run(w, init=init, leaf_steps=steps, sampler=1), F64_TOL, label="tile, far start, slice")


def test_tile_kernel_queues_chains_beyond_its_resident_slots_and_is_schedule_independent():
    w = W.small_logreg(40, 5, seed=8)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 9000, 3, 0.3, 5
    B = N()
    tgt = gpu_target(w)
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE, tgt=tgt)
    ids = np.array([0, 15, 16, 4097, 8191, 8192, 8999])
    assert_parity(g, ref_run(w, chain_ids=ids), F64_TOL, cols=ids, label="tile queue")
    small = gpu_run(w, variant=B.NUTS_VARIANT_TILE, tgt=tgt, n_chains=5)
    off = gpu_run(w, variant=B.NUTS_VARIANT_TILE, tgt=tgt, n_chains=33, first_chain=8000)
    again = gpu_run(w, variant=B.NUTS_VARIANT_TILE, tgt=tgt)
    for k in range(3):
        assert np.array_equal(g[k][:, :5], small[k])
        assert np.array_equal(g[k][:, 8000:8033], off[k])
        assert np.array_equal(g[k], again[k])


# ------------------------------------------------------------------ grid kernels (binary32, chip-wide GEMM per round)

def f32_parity(g, r, min_agree=0.99, min_chains=0.95):
    """binary32: a decision that falls the other way in rounding changes a chain's whole future, so integer outputs
    are compared as a rate, and states on the chains whose decisions all agree (per coordinate, see state_error).
    Measured over every binary32 comparison of this file (27 of them, 3 to 256 chains, up to 20 iterations): all
    integer outputs agree and no chain leaves the oracle's decisions; largest state error 2.5e-6.  The floors below
    leave room for one flipped decision in a hundred, not more."""
    same = (g[1] == r[1]) & (g[2] == r[2])
    ok = same.all(axis=0)
    err = state_error(g[0][:, ok], r[0][:, ok])
    report("f32", agree=float(same.mean()), chains_ok=float(ok.mean()), n_chains=int(ok.size), err=err)
    assert same.mean() >= min_agree, f"only {same.mean():.2%} of integer outputs agree"
    assert ok.sum() >= max(1, int(min_chains * ok.size)), f"only {ok.mean():.2%} of the chains never left the oracle's decisions"
    assert err <= F32_TOL, err


@pytest.mark.parametrize("n_data,dim,n_chains", [(5, 2, 3), (100, 7, 8), (1000, 33, 40), (3000, 100, 64),
                                                 (257, 128, 9), (4100, 65, 256), (31, 96, 5),
                                                 (600, 20, 129), (900, 40, 131), (2000, 100, 200),
                                                 (500, 72, 33), (700, 104, 17), (300, 97, 10)])
def test_logreg_f32_grid_kernels_ragged_shapes(n_data, dim, n_chains):
    w = W.small_logreg(n_data, dim, seed=200 + n_data, dtype=np.float32)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = n_chains, 6, 0.15 / np.sqrt(max(n_data, 1) / 10), 6
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_GRID)
    assert g[3]["variant"] == B.NUTS_VARIANT_GRID
    r = ref_run(w)
    check_invariants(w, g[1], g[2])
    f32_parity(g, r)
    assert g[3]["leaf_slots_useful"] == g[2].sum() and g[3]["extra_grad_evals"] == n_chains


def test_config4_large_logreg_f32_grid_kernels():
    w = W.make(4, n_chains=8, n_iters=10)
    B = N()
    g = gpu_run(w)
    assert g[3]["variant"] == B.NUTS_VARIANT_GRID      # chosen automatically for a chip-sized gradient
    f32_parity(g, ref_run(w))


def test_grid_kernels_are_schedule_independent_and_deterministic():
    w = W.small_logreg(2000, 20, seed=77, dtype=np.float32)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 100, 5, 0.02, 6
    B = N()
    tgt = gpu_target(w)
    a = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt)
    b = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt)
    c = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt, n_chains=37)
    o = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt, n_chains=10, first_chain=50)
    for k in range(3):
        assert np.array_equal(a[k], b[k])
        assert np.array_equal(a[k][:, :37], c[k])
        assert np.array_equal(a[k][:, 50:60], o[k])


def test_grid_kernels_two_sets_of_chains_equal_one_set():
    # beyond 128 chains the grid kernels step two sets of chains on two streams: same bytes as one set at a time
    w = W.small_logreg(1500, 30, seed=78, dtype=np.float32)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 200, 5, 0.03, 6
    B = N()
    tgt = gpu_target(w)
    a = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt)
    b = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt)
    lo = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt, n_chains=128)
    hi = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt, n_chains=72, first_chain=128)
    for k in range(3):
        assert np.array_equal(a[k], b[k])
        assert np.array_equal(a[k][:, :128], lo[k])
        assert np.array_equal(a[k][:, 128:], hi[k])
    st = a[3]
    assert st["leaf_slots_useful"] == a[2].sum() and st["leaf_slots_issued"] >= st["leaf_slots_useful"]


@pytest.mark.parametrize("n_chains", [700, 1300])
def test_grid_kernels_many_sets_and_queued_chains(n_chains):
    # 700 chains: six sets on four streams; 1300: more chains than the 1024 resident slots, the rest are queued
    w = W.small_logreg(800, 12, seed=79, dtype=np.float32)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = n_chains, 4, 0.05, 5
    B = N()
    tgt = gpu_target(w)
    a = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt)
    assert a[3]["variant"] == B.NUTS_VARIANT_GRID
    check_invariants(w, a[1], a[2])
    f32_parity(a, ref_run(w))
    assert a[3]["leaf_slots_useful"] == a[2].sum() and a[3]["extra_grad_evals"] == n_chains
    # which slot takes which chain depends on timing; the chains' results do not
    b = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt)
    c = gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt, n_chains=300)
    for k in range(3):
        assert np.array_equal(a[k], b[k])
        assert np.array_equal(a[k][:, :300], c[k])
    both_schedules(w, B.NUTS_VARIANT_GRID)


# ------------------------------------------------------------------ independence of the schedule

def test_chain_results_do_not_depend_on_batch_size_or_slot():
    """Section 2 of the paper: a batch member's execution is what it would be alone."""
    w = W.make(3, n_chains=300, n_iters=6)
    tgt = gpu_target(w)
    B = N()
    big = gpu_run(w, variant=B.NUTS_VARIANT_WAVE, tgt=tgt)
    small = gpu_run(w, variant=B.NUTS_VARIANT_WAVE, tgt=tgt, n_chains=7)
    off = gpu_run(w, variant=B.NUTS_VARIANT_WAVE, tgt=tgt, n_chains=20, first_chain=100)
    again = gpu_run(w, variant=B.NUTS_VARIANT_WAVE, tgt=tgt)
    for k in range(3):
        assert np.array_equal(big[k][:, :7], small[k])
        assert np.array_equal(big[k][:, 100:120], off[k])
        assert np.array_equal(big[k], again[k])


def test_more_chains_than_resident_slots_are_queued():
    w = W.Workload("queue", W.STD_NORMAL, 8, np.dtype(np.float64), 20000, 2, 0.4, 5, seed=11)
    g = gpu_run(w)
    ids = np.array([0, 1, 4999, 12345, 19999])
    assert_parity(g, ref_run(w, chain_ids=ids), F64_TOL, cols=ids, label="queued chains")
    assert g[3]["leaf_slots_useful"] == g[2].sum() and g[3]["extra_grad_evals"] == 20000


def test_null_outputs_are_allowed():
    import torch
    B = N()
    w = W.make(1)
    tgt = gpu_target(w)
    d = torch.empty((w.n_iters, w.n_chains), dtype=torch.int32, device="cuda")
    B._check(B.lib().nuts_sample(tgt.handle, w.n_chains, w.n_iters, w.step_size, w.max_tree_depth, w.seed,
                                 None, d.data_ptr(), None))
    torch.cuda.synchronize()
    assert np.array_equal(d.cpu().numpy(), ref_run(w)[1])


def test_runs_on_a_caller_stream():
    import torch
    B = N()
    w = W.make(1)
    s = torch.cuda.Stream()
    B.nuts_set_stream(s)
    try:
        with torch.cuda.stream(s):
            g = gpu_run(w)
    finally:
        B.nuts_set_stream(None)
    assert_parity(g, ref_run(w), F64_TOL, label="stream")


def test_grid_kernels_on_a_caller_stream_back_to_back_calls():
    # the grid path forks to streams of its own and joins them to the caller's: calls of different sizes in a row
    # (the workspace grows between them) on a caller's stream must equal the same calls on the default stream
    import torch
    B = N()
    w = W.small_logreg(700, 10, seed=81, dtype=np.float32)
    w.n_iters, w.step_size, w.max_tree_depth = 4, 0.05, 5
    tgt = gpu_target(w)
    ref = [gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=gpu_target(w), n_chains=c) for c in (40, 600, 130)]
    s = torch.cuda.Stream()
    B.nuts_set_stream(s)
    try:
        with torch.cuda.stream(s):
            got = [gpu_run(w, variant=B.NUTS_VARIANT_GRID, tgt=tgt, n_chains=c) for c in (40, 600, 130)]
    finally:
        B.nuts_set_stream(None)
    for a, b in zip(ref, got):
        for k in range(3):
            assert np.array_equal(a[k], b[k])


# ------------------------------------------------------------------ several leapfrog steps per leaf (Section 4.1 uses 4)

def check_leaf_invariants(w, d, n, k):
    leaves = n // k
    assert (n % k == 0).all()
    assert (leaves >= 2 ** (d.astype(np.int64) - 1)).all() and (leaves <= 2 ** d.astype(np.int64) - 1).all()


@pytest.mark.parametrize("k", [2, 4, 7])
@pytest.mark.parametrize("variant", [1, 3])
def test_leaf_steps_std_normal_and_diag(variant, k):
    w = W.Workload(f"std_k{k}", W.STD_NORMAL, 67, np.dtype(np.float64), 9, 12, 0.35 / k, 7, seed=50 + k)
    g = gpu_run(w, variant=variant, leaf_steps=k)
    assert g[3]["variant"] == variant and g[3]["leaf_slots_useful"] == g[2].sum()
    check_leaf_invariants(w, g[1], g[2], k)
    assert_parity(g, ref_run(w, leaf_steps=k), F64_TOL, label=w.name)
    sig = 10.0 ** np.random.default_rng(k).uniform(-1, 1, 130)
    w = W.Workload(f"diag_k{k}", W.GAUSS_DIAG, 130, np.dtype(np.float64), 6, 8, 0.05 / k, 8, seed=7, scales=sig)
    assert_parity(gpu_run(w, variant=variant, leaf_steps=k), ref_run(w, leaf_steps=k), F64_TOL, label=w.name)


def test_leaf_steps_dense_gaussian_config2_paper_setting():
    """Configuration 2 at the paper's own leaf size: 4 leapfrog steps per leaf."""
    w = W.make(2, n_chains=24, n_iters=20)
    w.step_size = w.step_size / 2
    g = gpu_run(w, leaf_steps=4)
    check_leaf_invariants(w, g[1], g[2], 4)
    assert_parity(g, ref_run(w, leaf_steps=4), F64_TOL, label="config 2, 4 steps per leaf")


@pytest.mark.parametrize("k", [2, 4])
@pytest.mark.parametrize("n_data,dim", [(65, 17), (1000, 25), (129, 32)])
def test_leaf_steps_logreg_tile_and_wave_kernels(n_data, dim, k):
    w = W.small_logreg(n_data, dim, seed=100 + n_data)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 21, 12, 0.3 / k / np.sqrt(max(n_data, 1) / 10), 7
    B = N()
    r = ref_run(w, leaf_steps=k)
    assert len(np.unique(r[1])) >= 2
    for variant in (B.NUTS_VARIANT_TILE, B.NUTS_VARIANT_WAVE):
        g = gpu_run(w, variant=variant, leaf_steps=k)
        assert g[3]["variant"] == variant and g[3]["leaf_slots_useful"] == g[2].sum()
        check_leaf_invariants(w, g[1], g[2], k)
        assert_parity(g, r, F64_TOL, label=f"{w.name} variant {variant} k={k}")


def test_leaf_steps_config3_tile_kernel_at_full_chain_count():
    w = W.make(3, n_iters=20)
    w.step_size = w.step_size / 2
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE, leaf_steps=4)
    check_leaf_invariants(w, g[1], g[2], 4)
    ids = np.concatenate([np.arange(8), np.random.default_rng(2).choice(4096, 24, replace=False), [4095]])
    assert_parity(g, ref_run(w, chain_ids=ids, leaf_steps=4), F64_TOL, cols=ids, label="config 3, 4 steps per leaf")


def test_leaf_steps_with_divergences_tile_kernel():
    w = W.small_logreg(50, 4, seed=6)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 20, 20, 0.45, 6
    B = N()
    init = np.random.default_rng(1).standard_normal((20, 4)) * 5
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE, init=init, leaf_steps=2)
    r = ref_run(w, init=init, leaf_steps=2)
    assert (r[2] // 2 != 2 ** r[1].astype(np.int64) - 1).sum() > 5
    assert_parity(g, r, F64_TOL, label="tile divergent k=2")


@pytest.mark.parametrize("n_data,dim,n_chains,k", [(100, 7, 8, 2), (1000, 33, 40, 4), (257, 128, 9, 3)])
def test_leaf_steps_logreg_f32_grid_kernels(n_data, dim, n_chains, k):
    w = W.small_logreg(n_data, dim, seed=200 + n_data, dtype=np.float32)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = n_chains, 6, 0.3 / k / np.sqrt(max(n_data, 1) / 10), 6
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_GRID, leaf_steps=k)
    assert g[3]["variant"] == B.NUTS_VARIANT_GRID and g[3]["leaf_slots_useful"] == g[2].sum()
    check_leaf_invariants(w, g[1], g[2], k)
    f32_parity(g, ref_run(w, leaf_steps=k))


def test_leaf_steps_argument_is_validated():
    B = N()
    t = B.Target(W.STD_NORMAL, 3, np.float64)
    for bad in (-1, 65):
        with pytest.raises(B.NutsError):
            B.nuts_sample(t, 2, 2, 0.1, 3, 1, leaf_steps=bad)


# ------------------------------------------------------------------ trajectory-synchronised schedule (Section 4.2)

def both_schedules(w, variant, **kw):
    B = N()
    tgt = gpu_target(w)
    free = gpu_run(w, variant=variant, tgt=tgt, schedule=B.NUTS_SCHEDULE_FREE, **kw)
    sync = gpu_run(w, variant=variant, tgt=tgt, schedule=B.NUTS_SCHEDULE_TRAJECTORY, **kw)
    assert free[3]["variant"] == sync[3]["variant"] == variant
    for a, b in zip(free[:3], sync[:3]):
        assert np.array_equal(a, b)             # the schedule must not show in the outputs
    n_chains, n_iters = free[1].shape[1], free[1].shape[0]
    assert free[3]["extra_grad_evals"] == n_chains
    assert sync[3]["extra_grad_evals"] == n_chains * n_iters
    assert sync[3]["leaf_slots_useful"] == free[3]["leaf_slots_useful"] == free[2].sum()
    return free, sync


@pytest.mark.parametrize("variant", [1, 3])
def test_schedules_agree_std_normal_and_diag(variant):
    w = W.Workload("std_sync", W.STD_NORMAL, 67, np.dtype(np.float64), 9, 12, 0.35, 7, seed=61)
    free, sync = both_schedules(w, variant)
    assert_parity(sync, ref_run(w), F64_TOL, label="std normal, trajectory schedule")
    sig = (10.0 ** np.random.default_rng(3).uniform(-1, 1, 300)).astype(np.float32)
    w = W.Workload("diag32_sync", W.GAUSS_DIAG, 300, np.dtype(np.float32), 10, 6, 0.05, 8, seed=17, scales=sig)
    both_schedules(w, variant)


def test_schedules_agree_dense_gaussian_and_occupancy_drops():
    """Figure 7's point: waiting at trajectory boundaries wastes gradient slots, batching across them does not."""
    w = W.make(2, n_chains=64, n_iters=10)
    free, sync = both_schedules(w, 1)
    assert_parity(sync, ref_run(w), F64_TOL, label="config 2, trajectory schedule")
    nl = free[2].astype(np.int64)
    # one chain per slot: the launch lasts as long as its busiest chain
    want_sync = nl.sum() / (64 * (nl.max(axis=1) + 1).sum())
    want_free = nl.sum() / (64 * (nl.sum(axis=0) + 1).max())
    assert abs(sync[3]["occupancy"] - want_sync) < 1e-12
    assert abs(free[3]["occupancy"] - want_free) < 1e-12
    assert sync[3]["occupancy"] < free[3]["occupancy"]


@pytest.mark.parametrize("n_data,dim", [(65, 17), (1000, 25)])
def test_schedules_agree_logreg_tile_and_wave_kernels(n_data, dim):
    w = W.small_logreg(n_data, dim, seed=100 + n_data)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 37, 9, 0.15 / np.sqrt(max(n_data, 1) / 10), 7
    B = N()
    r = ref_run(w)
    for variant in (B.NUTS_VARIANT_TILE, B.NUTS_VARIANT_WAVE):
        free, sync = both_schedules(w, variant)
        assert_parity(sync, r, F64_TOL, label=f"logreg variant {variant}, trajectory schedule")
    assert sync[3]["occupancy"] <= 1.0


def test_schedules_agree_logreg_f32_grid_kernels():
    w = W.small_logreg(1000, 33, seed=1200, dtype=np.float32)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 12, 5, 0.015, 6
    B = N()
    both_schedules(w, B.NUTS_VARIANT_GRID)


def test_trajectory_schedule_with_leaf_steps_init_states_offsets_and_no_state_output():
    import torch
    B = N()
    w = W.small_logreg(200, 6, seed=77)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 19, 7, 0.05, 6
    init = np.random.default_rng(4).standard_normal((19, 6))
    free, sync = both_schedules(w, B.NUTS_VARIANT_TILE, init=init, first_chain=1000, leaf_steps=3)
    tgt = gpu_target(w)
    s, d, n = B.nuts_sample(tgt, 19, 7, w.step_size, w.max_tree_depth, w.seed, variant=B.NUTS_VARIANT_TILE,
                            init_states=torch.as_tensor(init).cuda(), first_chain=1000, leaf_steps=3,
                            schedule=B.NUTS_SCHEDULE_TRAJECTORY, want_states=False)
    torch.cuda.synchronize()
    assert s is None
    assert np.array_equal(d.cpu().numpy(), free[1]) and np.array_equal(n.cpu().numpy(), free[2])
    with pytest.raises(B.NutsError):
        B.nuts_sample(tgt, 2, 2, 0.1, 3, 1, schedule=2)


# ------------------------------------------------------------------ slice-sampling form (the published algorithm)

SLICE = 1


@pytest.mark.parametrize("variant", [1, 3])
def test_slice_sampler_std_normal_diag_and_deep_trees(variant):
    w = W.Workload("std_slice", W.STD_NORMAL, 67, np.dtype(np.float64), 9, 12, 0.35, 7, seed=71)
    g = gpu_run(w, variant=variant, sampler=SLICE)
    r = ref_run(w, sampler=SLICE)
    assert g[3]["variant"] == variant
    assert_parity(g, r, F64_TOL, label="std normal, slice")
    assert not np.array_equal(r[0], ref_run(w)[0])
    sig = 10.0 ** np.random.default_rng(9).uniform(-1, 1, 130)
    w = W.Workload("diag_slice", W.GAUSS_DIAG, 130, np.dtype(np.float64), 6, 8, 0.05, 8, seed=7, scales=sig)
    assert_parity(gpu_run(w, variant=variant, sampler=SLICE), ref_run(w, sampler=SLICE), F64_TOL, label="diag, slice")
    w = W.Workload("deep_slice", W.STD_NORMAL, 2, np.dtype(np.float64), 5, 3, 0.004, 10, seed=8)
    r = ref_run(w, sampler=SLICE)
    assert r[1].max() == 10 and r[2].max() == 1023
    assert_parity(gpu_run(w, variant=variant, sampler=SLICE), r, F64_TOL, label="deep trees, slice")


@pytest.mark.parametrize("variant", [1, 3])
def test_slice_sampler_divergences_and_non_finite_energy(variant):
    init = np.random.default_rng(0).standard_normal((12, 2)) * np.array([1.0, 40.0])
    w = W.Workload("div_slice", W.STD_NORMAL, 2, np.dtype(np.float64), 12, 30, 1.75, 5, seed=5)
    r = ref_run(w, init=init, sampler=SLICE)
    assert (r[2] != 2 ** r[1].astype(np.int64) - 1).sum() > 5
    assert_parity(gpu_run(w, init=init, variant=variant, sampler=SLICE), r, F64_TOL, label="divergent, slice")
    init = np.full((3, 2), 1e200)
    w = W.Workload("inf_slice", W.STD_NORMAL, 2, np.dtype(np.float64), 3, 4, 0.5, 4, seed=2)
    g = gpu_run(w, init=init, variant=variant, sampler=SLICE)
    r = ref_run(w, init=init, sampler=SLICE)
    assert (g[1] == 1).all() and np.array_equal(g[1], r[1]) and np.array_equal(g[2], r[2]) and np.array_equal(g[0], r[0])


def test_slice_sampler_dense_gaussian_config2():
    w = W.make(2, n_chains=24, n_iters=20)
    assert_parity(gpu_run(w, sampler=SLICE), ref_run(w, sampler=SLICE), F64_TOL, label="config 2, slice")
    assert_parity(gpu_run(w, sampler=SLICE, leaf_steps=4), ref_run(w, sampler=SLICE, leaf_steps=4), F64_TOL,
                  label="config 2, slice, 4 steps per leaf (the paper's setting)")


@pytest.mark.parametrize("n_data,dim", [(5, 2), (65, 17), (1000, 25), (129, 32)])
def test_slice_sampler_logreg_tile_and_wave_kernels(n_data, dim):
    w = W.small_logreg(n_data, dim, seed=100 + n_data)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 21, 12, 0.15 / np.sqrt(max(n_data, 1) / 10), 7
    B = N()
    r = ref_run(w, sampler=SLICE)
    for variant in (B.NUTS_VARIANT_TILE, B.NUTS_VARIANT_WAVE):
        g = gpu_run(w, variant=variant, sampler=SLICE)
        assert g[3]["variant"] == variant and g[3]["leaf_slots_useful"] == g[2].sum()
        assert_parity(g, r, F64_TOL, label=f"{w.name} variant {variant}, slice")
    r = ref_run(w, sampler=SLICE, leaf_steps=2)
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE, sampler=SLICE, leaf_steps=2, schedule=B.NUTS_SCHEDULE_TRAJECTORY)
    assert_parity(g, r, F64_TOL, label=f"{w.name} tile, slice, 2 steps per leaf, trajectory schedule")


def test_slice_sampler_config3_tile_kernel_at_full_chain_count():
    w = W.make(3, n_iters=30)
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_TILE, sampler=SLICE)
    check_invariants(w, g[1], g[2])
    ids = np.concatenate([np.arange(8), np.random.default_rng(3).choice(4096, 32, replace=False), [4095]])
    assert_parity(g, ref_run(w, chain_ids=ids, sampler=SLICE), F64_TOL, cols=ids, label="config 3, slice")


def test_slice_sampler_tile_kernel_divergences_and_deep_trees():
    B = N()
    w = W.small_logreg(50, 4, seed=6)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 20, 20, 0.6, 6
    init = np.random.default_rng(1).standard_normal((20, 4)) * 5
    r = ref_run(w, init=init, sampler=SLICE)
    assert (r[2] != 2 ** r[1].astype(np.int64) - 1).sum() > 5
    assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_TILE, init=init, sampler=SLICE), r, F64_TOL, label="tile divergent, slice")
    w = W.small_logreg(30, 3, seed=4)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 18, 2, 0.0005, 12
    r = ref_run(w, sampler=SLICE)
    assert r[1].max() == 12
    assert_parity(gpu_run(w, variant=B.NUTS_VARIANT_TILE, sampler=SLICE), r, F64_TOL, label="tile depth 12, slice")


def test_slice_sampler_logreg_f32_grid_kernels_and_bad_argument():
    w = W.small_logreg(1000, 33, seed=1200, dtype=np.float32)
    w.n_chains, w.n_iters, w.step_size, w.max_tree_depth = 40, 6, 0.015, 6
    B = N()
    g = gpu_run(w, variant=B.NUTS_VARIANT_GRID, sampler=SLICE)
    assert g[3]["variant"] == B.NUTS_VARIANT_GRID
    f32_parity(g, ref_run(w, sampler=SLICE))
    with pytest.raises(B.NutsError):
        B.nuts_sample(gpu_target(w), 2, 2, 0.1, 3, 1, sampler=2)


# ------------------------------------------------------------------ dense-Gaussian register kernel (matrix in LDS)

DENSE = 5


@pytest.mark.parametrize("dim", [1, 2, 3, 63, 64, 65, 100, 127, 128])
def test_dense_register_kernel_ragged_dimensions(dim):
    w = W.Workload(f"dense_d{dim}", W.GAUSS_DENSE, dim, np.dtype(np.float64), 7, 10, 0.2, 7, seed=6,
                   precision=W.random_spd_precision(dim, 3))
    g = gpu_run(w, variant=DENSE)
    assert g[3]["variant"] == DENSE and g[3]["leaf_slots_useful"] == g[2].sum() and g[3]["extra_grad_evals"] == 7
    assert_parity(g, ref_run(w), F64_TOL, label=w.name)
    auto = gpu_run(w)
    assert auto[3]["variant"] == DENSE
    for a, b in zip(g[:3], auto[:3]):
        assert np.array_equal(a, b)


def test_dense_register_kernel_config2_full_chain_count_and_queueing():
    w = W.make(2, n_iters=50)
    g = gpu_run(w)
    assert g[3]["variant"] == DENSE
    check_invariants(w, g[1], g[2])
    ids = np.array([0, 1, 2, 3, 500, 777, 1022, 1023])
    assert_parity(g, ref_run(w, chain_ids=ids), F64_TOL, cols=ids, label="config 2, dense kernel")
    w = W.make(2, n_chains=5000, n_iters=2)          # more chains than resident slots: the queue refills them
    g = gpu_run(w)
    ids = np.array([0, 1023, 1024, 2047, 2048, 4999])
    assert_parity(g, ref_run(w, chain_ids=ids), F64_TOL, cols=ids, label="config 2, queued chains")


def test_dense_register_kernel_options_and_limits():
    B = N()
    w = W.make(2, n_chains=24, n_iters=12)
    for kw in (dict(leaf_steps=4), dict(sampler=SLICE), dict(sampler=SLICE, leaf_steps=2)):
        g = gpu_run(w, variant=DENSE, **kw)
        assert_parity(g, ref_run(w, **kw), F64_TOL, label=f"config 2 dense kernel {kw}")
    free, sync = both_schedules(w, DENSE)
    init = np.random.default_rng(3).standard_normal((24, w.dim)) * 10      # far out, near the stability limit
    w.step_size = 0.44
    g = gpu_run(w, variant=DENSE, init=init)
    r = ref_run(w, init=init)
    assert (r[2] != 2 ** r[1].astype(np.int64) - 1).sum() > 5
    assert_parity(g, r, F64_TOL, label="config 2 dense kernel, divergent")
    # much further out: leaves land thousands below the starting energy, and the unit of the weights moves
    init = np.random.default_rng(4).standard_normal((24, w.dim)) * 60
    w.step_size = 0.3
    assert_parity(gpu_run(w, variant=DENSE, init=init), ref_run(w, init=init), F64_TOL, label="config 2 dense kernel, far start")
    big = W.Workload("dense_d129", W.GAUSS_DENSE, 129, np.dtype(np.float64), 3, 2, 0.2, 4, seed=6,
                     precision=W.random_spd_precision(129, 3))
    with pytest.raises(B.NutsError):
        gpu_run(big, variant=DENSE)
    assert gpu_run(big)[3]["variant"] == B.NUTS_VARIANT_WAVE


def test_dense_register_kernel_f32():
    P = W.random_spd_precision(70, 5).astype(np.float32)
    w = W.Workload("dense32", W.GAUSS_DENSE, 70, np.dtype(np.float32), 12, 6, 0.2, 6, seed=9, precision=P)
    g = gpu_run(w, variant=DENSE)
    assert g[3]["variant"] == DENSE
    f32_parity(g, ref_run(w))


# ------------------------------------------------------------------ quad kernel (four chains per wavefront, P theta on MFMA blocks)

QUAD = 6


@pytest.mark.parametrize("dim,n_chains", [(1, 1), (2, 3), (3, 4), (15, 5), (16, 16), (17, 21), (63, 33), (64, 7), (65, 64),
                                           (100, 37), (127, 9), (128, 70)])
def test_quad_kernel_ragged_dimensions_and_chain_counts(dim, n_chains):
    w = W.Workload(f"quad_d{dim}", W.GAUSS_DENSE, dim, np.dtype(np.float64), n_chains, 10, 0.2, 7, seed=6 + dim,
                   precision=W.random_spd_precision(dim, 3))
    g = gpu_run(w, variant=QUAD)
    assert g[3]["variant"] == QUAD and g[3]["leaf_slots_useful"] == g[2].sum() and g[3]["extra_grad_evals"] == n_chains
    r = ref_run(w)
    assert r[2].max() >= 3
    assert_parity(g, r, F64_TOL, label=w.name)
    dense = gpu_run(w, variant=DENSE)            # the two kernels sum in different orders: same integers, states to rounding
    assert np.array_equal(dense[1], g[1]) and np.array_equal(dense[2], g[2])


def test_quad_kernel_random_spd_d100_many_chains_queueing_and_independence():
    """The case the kernel is for: a correlated Gaussian whose precision is not banded, more chains than resident
    slots (256 compute units x 16), chosen automatically."""
    w = W.Workload("quad_spd_d100", W.GAUSS_DENSE, 100, np.dtype(np.float64), 6000, 4, 0.15, 8, seed=21,
                   precision=W.random_spd_precision(100, 7))
    tgt = gpu_target(w)
    g = gpu_run(w, tgt=tgt)
    assert g[3]["variant"] == QUAD
    check_invariants(w, g[1], g[2])
    assert np.isfinite(g[0]).all()
    ids = np.array([0, 1, 2, 3, 4, 15, 16, 4095, 4096, 4097, 5999])
    assert_parity(g, ref_run(w, chain_ids=ids), F64_TOL, cols=ids, label="quad, queued chains")
    st = g[3]
    assert st["leaf_slots_useful"] == g[2].sum() and st["leaf_slots_issued"] >= st["leaf_slots_useful"] + 6000
    small = gpu_run(w, variant=QUAD, tgt=tgt, n_chains=5)
    off = gpu_run(w, variant=QUAD, tgt=tgt, n_chains=33, first_chain=3000)
    again = gpu_run(w, tgt=tgt)
    for k in range(3):
        assert np.array_equal(g[k][:, :5], small[k])          # a chain's results do not depend on the batch it runs in
        assert np.array_equal(g[k][:, 3000:3033], off[k])
        assert np.array_equal(g[k], again[k])
    few = gpu_run(w, tgt=tgt, n_chains=100)                    # few chains: one chain per wavefront spreads them better
    assert few[3]["variant"] == DENSE


def test_quad_kernel_options_deep_trees_and_divergences():
    B = N()
    w = W.Workload("quad_opts", W.GAUSS_DENSE, 40, np.dtype(np.float64), 23, 8, 0.25, 7, seed=5,
                   precision=W.random_spd_precision(40, 2))
    for kw in (dict(leaf_steps=4), dict(sampler=SLICE), dict(sampler=SLICE, leaf_steps=2)):
        assert_parity(gpu_run(w, variant=QUAD, **kw), ref_run(w, **kw), F64_TOL, label=f"quad {kw}")
    both_schedules(w, QUAD)
    both_schedules(w, QUAD, sampler=SLICE, leaf_steps=3)
    # deep trees up to the depth limit of the kernel
    w.step_size, w.max_tree_depth, w.n_iters, w.n_chains = 0.004, 10, 2, 6
    r = ref_run(w)
    assert r[1].max() == 10 and r[2].max() == 1023
    assert_parity(gpu_run(w, variant=QUAD), r, F64_TOL, label="quad deep")
    w.max_tree_depth, w.n_iters = 12, 1
    assert_parity(gpu_run(w, variant=QUAD), ref_run(w), F64_TOL, label="quad depth 12")
    w.max_tree_depth = 13
    with pytest.raises(B.NutsError):
        gpu_run(w, variant=QUAD)
    # far out and near the stability limit: divergent leaves, early exits, non-finite states
    w.step_size, w.max_tree_depth, w.n_iters, w.n_chains = 0.9, 6, 12, 20
    init = np.random.default_rng(3).standard_normal((20, w.dim)) * 10
    init[3] = 1e200
    init[7] = np.inf
    g = gpu_run(w, variant=QUAD, init=init)
    r = ref_run(w, init=init)
    assert (r[2] != 2 ** r[1].astype(np.int64) - 1).sum() > 5
    assert np.array_equal(np.isfinite(g[0]), np.isfinite(r[0]))
    assert np.array_equal(g[1], r[1]) and np.array_equal(g[2], r[2])
    fin = np.isfinite(r[0]).all(axis=(0, 2))
    assert state_error(g[0][:, fin], r[0][:, fin]) < F64_TOL
    f32 = W.Workload("quad_f32", W.GAUSS_DENSE, 8, np.dtype(np.float32), 4, 2, 0.2, 4, seed=1,
                     precision=W.random_spd_precision(8, 1).astype(np.float32))
    with pytest.raises(B.NutsError):
        gpu_run(f32, variant=QUAD)


# ------------------------------------------------------------------ the launches bench.py times, at full size

def full_size_run(cfg, **kw):
    """The exact launch of the benchmark (all chains, all iterations); only slices leave the GPU."""
    import torch
    B = N()
    w = W.make(cfg)
    tgt = gpu_target(w)
    s, d, n = B.nuts_sample(tgt, w.n_chains, w.n_iters, w.step_size, w.max_tree_depth, w.seed, **kw)
    torch.cuda.synchronize()
    return w, s, d, n, B.nuts_get_stats(tgt)


def test_config3_full_size_launch_first_50_iterations_and_invariants_everywhere():
    import torch
    w, s, d, n, st = full_size_run(3)
    assert st["variant"] == N().NUTS_VARIANT_TILE and st["leaf_slots_useful"] == int(n.sum().item())
    assert st["occupancy"] > 0.9
    dd, nn = d.to(torch.int64), n.to(torch.int64)
    assert bool(((dd >= 1) & (dd <= w.max_tree_depth) & (nn >= 2 ** (dd - 1)) & (nn <= 2 ** dd - 1)).all())
    assert bool(torch.isfinite(s).all())
    ids = np.concatenate([np.arange(4), np.random.default_rng(11).choice(4096, 20, replace=False), [4095]])
    r = ref_run(w, chain_ids=ids, n_iters=50)
    t = torch.as_tensor(ids).cuda()
    g = (s[:50][:, t].cpu().numpy(), d[:50][:, t].cpu().numpy(), n[:50][:, t].cpu().numpy())
    assert_parity(g, r, F64_TOL, label="config 3 at full size, first 50 iterations")
    # the sample itself: posterior means of all chains agree across two halves of the chains
    late = s[200:]
    a, b = late[:, :2048].mean(dim=(0, 1)), late[:, 2048:].mean(dim=(0, 1))
    assert float((a - b).abs().max()) < 0.02


def test_config2_full_size_launch_first_50_iterations():
    import torch
    w, s, d, n, st = full_size_run(2)
    assert st["variant"] == DENSE
    ids = np.array([0, 1, 511, 512, 1023])
    r = ref_run(w, chain_ids=ids, n_iters=50)
    t = torch.as_tensor(ids).cuda()
    g = (s[:50][:, t].cpu().numpy(), d[:50][:, t].cpu().numpy(), n[:50][:, t].cpu().numpy())
    assert_parity(g, r, F64_TOL, label="config 2 at full size, first 50 iterations")
    x = s[300:].reshape(-1, w.dim)
    cov = torch.cov(x.T).cpu().numpy()
    want = 0.9 ** np.abs(np.subtract.outer(np.arange(w.dim), np.arange(w.dim)))
    assert np.abs(cov - want).max() < 0.08 and float(x.mean(dim=0).abs().max()) < 0.05


def test_config4_full_size_launch_first_10_iterations_binary32():
    import torch
    w, s, d, n, st = full_size_run(4)
    assert st["variant"] == N().NUTS_VARIANT_GRID
    ids = np.arange(8)
    r = ref_run(w, chain_ids=ids, n_iters=10)
    g = (s[:10, :8].cpu().numpy(), d[:10, :8].cpu().numpy(), n[:10, :8].cpu().numpy())
    f32_parity(g, r)
    assert bool(torch.isfinite(s).all())


def test_config5_full_size_launch_first_20_iterations_binary32_and_invariants_everywhere():
    """The launch bench.py times on configuration 5: 16384 chains x 500 iterations, chains beyond the resident slots
    taken from the queue.  Sampled chains against the oracle over their first 20 iterations, per coordinate (the
    scales span four decades); structural invariants and finiteness over everything; the sample itself against the
    target's standard deviations."""
    import torch
    w, s, d, n, st = full_size_run(5)
    assert st["variant"] == N().NUTS_VARIANT_ELEM and st["leaf_slots_useful"] == int(n.sum().item())
    dd, nn = d.to(torch.int64), n.to(torch.int64)
    assert bool(((dd >= 1) & (dd <= w.max_tree_depth) & (nn >= 2 ** (dd - 1)) & (nn <= 2 ** dd - 1)).all())
    assert bool(torch.isfinite(s).all())
    ids = np.concatenate([np.arange(4), np.random.default_rng(5).choice(16384, 27, replace=False), [16383]])
    r = ref_run(w, chain_ids=ids, n_iters=20)
    t = torch.as_tensor(ids).cuda()
    g = (s[:20][:, t].cpu().numpy(), d[:20][:, t].cpu().numpy(), n[:20][:, t].cpu().numpy())
    f32_parity(g, r)
    # late iterations, a slice of the chains: every coordinate's spread is its sigma (trajectories of at most 1023 steps
    # of 0.01 do not cross the widest coordinates in one iteration, so those are still narrower than their sigma)
    x = s[300::20, ::8].reshape(-1, w.dim).to(torch.float64)
    ratio = (x.std(dim=0).cpu().numpy() / w.scales.astype(np.float64))
    narrow = w.scales < 1.0
    assert np.abs(ratio[narrow] - 1.0).max() < 0.1 and (ratio <= 1.1).all()
    del s, x


# ------------------------------------------------------------------ option matrix: every kernel x sampler x leaf size x schedule

def _matrix_cases():
    rng = np.random.default_rng(2024)
    cases = []
    for variant, kind in [(1, "std"), (3, "std"), (1, "diag"), (3, "diag"), (1, "dense"), (5, "dense"), (1, "logreg"),
                          (2, "logreg"), (4, "logreg32")]:
        for rep in range(4):
            cases.append((variant, kind, int(rng.integers(0, 2)), int(rng.choice([1, 2, 3, 5])), int(rng.integers(0, 2)),
                          int(rng.integers(1, 40)), int(rng.integers(1, 30)), int(rng.integers(0, 10**6))))
    return cases


@pytest.mark.parametrize("variant,kind,sampler,k,schedule,dim,n_chains,seed", _matrix_cases())
def test_option_matrix(variant, kind, sampler, k, schedule, dim, n_chains, seed):
    rng = np.random.default_rng(seed)
    n_iters, depth = 6, 6
    if kind == "std":
        w = W.Workload("m_std", W.STD_NORMAL, dim, np.dtype(np.float64), n_chains, n_iters, 0.5 / k, depth, seed=seed)
    elif kind == "diag":
        w = W.Workload("m_diag", W.GAUSS_DIAG, dim, np.dtype(np.float64), n_chains, n_iters, 0.1 / k, depth, seed=seed,
                       scales=10.0 ** rng.uniform(-0.5, 0.5, dim))
    elif kind == "dense":
        w = W.Workload("m_dense", W.GAUSS_DENSE, dim, np.dtype(np.float64), n_chains, n_iters, 0.3 / k, depth, seed=seed,
                       precision=W.random_spd_precision(dim, seed % 7))
    else:
        dim = min(dim, 32)
        n_data = int(rng.integers(1, 300))
        w = W.small_logreg(n_data, dim, seed=seed, dtype=np.float32 if kind == "logreg32" else np.float64)
        w.n_chains, w.n_iters, w.max_tree_depth = n_chains, n_iters, depth
        w.step_size = 0.3 / k / np.sqrt(max(n_data, 10) / 10)
        w.seed = seed
    g = gpu_run(w, variant=variant, sampler=sampler, leaf_steps=k, schedule=schedule)
    r = ref_run(w, sampler=sampler, leaf_steps=k)
    assert g[3]["variant"] == variant
    if kind == "logreg32":
        f32_parity(g, r)
    else:
        assert_parity(g, r, F64_TOL, label=f"{kind} v{variant} sampler={sampler} k={k} schedule={schedule} d={w.dim}")


def banded_spd(dim, half, seed):
    """A symmetric positive definite matrix that is exactly zero beyond `half` off-diagonals."""
    rng = np.random.default_rng(seed)
    P = np.zeros((dim, dim))
    for k in range(1, half + 1):
        v = rng.uniform(-0.4, 0.4, dim - k) if dim > k else np.zeros(0)
        P += np.diag(v, k) + np.diag(v, -k)
    return P + np.diag(np.abs(P).sum(axis=1) + rng.uniform(0.5, 2.0, dim))


@pytest.mark.parametrize("dim,half", [(1, 0), (2, 1), (9, 4), (100, 1), (100, 4), (128, 3), (127, 5), (40, 39)])
def test_dense_register_kernel_banded_and_nearly_banded_matrices(dim, half):
    """Up to four off-diagonals the kernel keeps the band in registers; beyond that it falls back to the
    matrix in LDS.  Both must match the oracle's dense sums."""
    half = min(half, dim - 1)
    w = W.Workload(f"band_d{dim}_h{half}", W.GAUSS_DENSE, dim, np.dtype(np.float64), 9, 10, 0.25, 7, seed=dim + half,
                   precision=banded_spd(dim, half, seed=dim))
    g = gpu_run(w, variant=DENSE)
    assert g[3]["variant"] == DENSE
    r = ref_run(w)
    assert r[2].max() >= 3
    assert_parity(g, r, F64_TOL, label=w.name)
    wave = gpu_run(w, variant=1)
    assert np.array_equal(wave[1], g[1]) and np.array_equal(wave[2], g[2])


def test_dense_register_kernel_banded_f32_and_options():
    P = banded_spd(60, 2, seed=3).astype(np.float32)
    w = W.Workload("band32", W.GAUSS_DENSE, 60, np.dtype(np.float32), 12, 6, 0.2, 6, seed=9, precision=P)
    f32_parity(gpu_run(w, variant=DENSE), ref_run(w))
    w = W.make(2, n_chains=24, n_iters=12)        # the AR(1) precision of configuration 2 is tridiagonal
    for kw in (dict(leaf_steps=4), dict(sampler=SLICE), dict(sampler=SLICE, leaf_steps=2)):
        assert_parity(gpu_run(w, variant=DENSE, **kw), ref_run(w, **kw), F64_TOL, label=f"banded {kw}")
    both_schedules(w, DENSE)
