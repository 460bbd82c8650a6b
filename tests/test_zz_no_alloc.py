"""nuts_sample_static: the entry point that allocates nothing (workspace and counters in a static device array).
It runs the same kernels as nuts_sample_ex, so its outputs must equal that entry point's bit for bit: on two
calls in a row, the second with a smaller input (the array keeps the first call's contents), for every kernel
family it admits; runs that do not fit or would need an allocation are refused before anything is written."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _run(B, tgt, w, n_chains, n_iters, static, **kw):
    import torch
    tdt = torch.float64 if w.dtype.itemsize == 8 else torch.float32
    out = (torch.full((n_iters, n_chains, w.dim), float("nan"), dtype=tdt, device="cuda"),
           torch.full((n_iters, n_chains), -1, dtype=torch.int32, device="cuda"),
           torch.full((n_iters, n_chains), -1, dtype=torch.int32, device="cuda"))
    B.nuts_sample(tgt, n_chains, n_iters, w.step_size, w.max_tree_depth, w.seed, out=out, static_scratch=static, **kw)
    torch.cuda.synchronize()
    st = B.nuts_get_stats(tgt)
    return [t.cpu().numpy() for t in out], st


@pytest.mark.parametrize("config,big,small,kw", [
    (3, (96, 12), (40, 7), {}),                       # tile kernel (MFMA gradient)
    (3, (64, 6), (24, 4), {"variant": 1}),            # wave kernel
    (5, (48, 6), (16, 4), {}),                        # element-wise kernel
    (2, (64, 8), (12, 5), {}),                        # dense-Gaussian kernel
    (1, (4, 30), (3, 10), {}),                        # standard normal
    (3, (64, 6), (32, 3), {"leaf_steps": 3, "sampler": 1, "schedule": 1}),
])
def test_static_entry_point_equals_the_allocating_one_twice_in_a_row(config, big, small, kw):
    import paper_1910_11141_amd.binding as B
    from paper_1910_11141_amd import workloads
    w = workloads.make(config, n_chains=big[0], n_iters=big[1])
    tgt = B.Target(w.kind, w.dim, w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y, prior_scale=w.prior_scale)
    for n_chains, n_iters in (big, small):
        print(f"config {config} {kw} chains {n_chains} iters {n_iters}", flush=True)
        want, st_want = _run(B, tgt, w, n_chains, n_iters, False, **kw)
        got, st_got = _run(B, tgt, w, n_chains, n_iters, True, **kw)
        for a, b in zip(want, got):
            assert np.array_equal(a, b)
        assert (want[1] >= 1).all() and np.isfinite(want[0]).all()
        # (slots issued depend on which workgroup takes which chain from the queue, i.e. on timing)
        for key in ("leaf_slots_useful", "extra_grad_evals", "variant"):
            assert st_got[key] == st_want[key], key
        assert st_got["leaf_slots_issued"] >= st_got["leaf_slots_useful"]
        assert st_got["leaf_slots_useful"] == int(got[2].sum())


def test_static_entry_point_refuses_what_does_not_fit_or_would_allocate():
    import torch
    import paper_1910_11141_amd.binding as B
    from paper_1910_11141_amd import workloads
    # configuration 5 at full width needs gigabytes of tree storage
    w = workloads.make(5, n_chains=16384, n_iters=2)
    tgt = B.Target(w.kind, w.dim, w.dtype, scales=w.scales)
    out = (torch.zeros((2, 16384, w.dim), dtype=torch.float32, device="cuda"),
           torch.zeros((2, 16384), dtype=torch.int32, device="cuda"), torch.zeros((2, 16384), dtype=torch.int32, device="cuda"))
    with pytest.raises(B.NutsError) as e:
        B.nuts_sample(tgt, 16384, 2, w.step_size, w.max_tree_depth, w.seed, out=out, static_scratch=True)
    assert e.value.code == B.NUTS_E_UNSUPPORTED and "bytes of scratch" in str(e.value)
    torch.cuda.synchronize()
    assert int(out[1].abs().sum()) == 0 and float(out[0].abs().sum()) == 0.0      # nothing was written
    # the grid kernels own streams and pinned memory
    w = workloads.make(4, n_chains=8, n_iters=2)
    tgt = B.Target(w.kind, w.dim, w.dtype, X=w.X[:4096], y=w.y[:4096], prior_scale=w.prior_scale)
    with pytest.raises(B.NutsError) as e:
        B.nuts_sample(tgt, 8, 2, w.step_size, w.max_tree_depth, w.seed, static_scratch=True)
    assert e.value.code == B.NUTS_E_UNSUPPORTED
    # the trajectory schedule without a states buffer would need a carry buffer
    w = workloads.make(1)
    tgt = B.Target(w.kind, w.dim, w.dtype)
    with pytest.raises(B.NutsError) as e:
        B.nuts_sample(tgt, 4, 3, w.step_size, w.max_tree_depth, w.seed, want_states=False, schedule=1, static_scratch=True)
    assert e.value.code == B.NUTS_E_UNSUPPORTED
    # and the full headline configuration fits
    w = workloads.make(3, n_iters=3)
    tgt = B.Target(w.kind, w.dim, w.dtype, X=w.X, y=w.y, prior_scale=w.prior_scale)
    a = B.nuts_sample(tgt, w.n_chains, 3, w.step_size, w.max_tree_depth, w.seed, static_scratch=True)
    b = B.nuts_sample(tgt, w.n_chains, 3, w.step_size, w.max_tree_depth, w.seed)
    torch.cuda.synchronize()
    assert all(bool(torch.equal(x, y)) for x, y in zip(a, b))
