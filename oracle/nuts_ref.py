"""ctypes view of the CPU oracle (oracle/nuts_ref.c).

Test infrastructure: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py only.  The product package never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnuts_ref.so")

F32, F64 = 0, 1
STD_NORMAL, GAUSS_DENSE, GAUSS_DIAG, LOGREG = 0, 1, 2, 3
TAG_INIT, TAG_MOMENTUM, TAG_DIRECTION, TAG_SUBTREE, TAG_TOP, TAG_SLICE = 0, 1, 2, 3, 4, 5
MULTINOMIAL, SLICE = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no FMA contraction, generic x86-64)."""
    srcs = [os.path.join(_HERE, "nuts_ref.c"), os.path.join(_HERE, "nuts_ref_typed.inc")]
    if not force and os.path.exists(LIB_PATH) and all(
        os.path.getmtime(LIB_PATH) >= os.path.getmtime(s) for s in srcs
    ):
        return LIB_PATH
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-fPIC",
           "-shared", "-pthread", "-o", LIB_PATH, srcs[0], "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return LIB_PATH


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(LIB_PATH)
        L.nuts_ref_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
        L.nuts_ref_philox4x32_10.restype = None
        L.nuts_ref_draw.argtypes = [C.c_uint64] + [C.c_uint32] * 5 + [C.POINTER(C.c_uint32)]
        L.nuts_ref_draw.restype = None
        L.nuts_ref_uniform.argtypes = [C.c_uint32, C.c_uint32]
        L.nuts_ref_uniform.restype = C.c_double
        L.nuts_ref_normal_pair.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_double)]
        L.nuts_ref_normal_pair.restype = None
        L.nuts_ref_logaddexp.argtypes = [C.c_double, C.c_double]
        L.nuts_ref_logaddexp.restype = C.c_double
        tgt = [C.c_int, C.c_int, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_double]
        L.nuts_ref_logp_grad.argtypes = tgt + [C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
        L.nuts_ref_logp_grad.restype = C.c_int
        L.nuts_ref_leapfrog.argtypes = tgt + [C.c_void_p, C.c_void_p, C.c_double, C.c_int64, C.POINTER(C.c_double)]
        L.nuts_ref_leapfrog.restype = C.c_int
        L.nuts_ref_uturn_ok.argtypes = [C.c_int, C.c_int64] + [C.c_void_p] * 4
        L.nuts_ref_uturn_ok.restype = C.c_int
        L.nuts_ref_sample.argtypes = tgt + [C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_double, C.c_int32,
                                            C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
        L.nuts_ref_sample.restype = C.c_int
        L.nuts_ref_sample_k.argtypes = tgt + [C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_double, C.c_int32,
                                              C.c_int32, C.c_int32, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_int32]
        L.nuts_ref_sample_k.restype = C.c_int
        _lib = L
    return _lib


def philox(ctr, key) -> np.ndarray:
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    lib().nuts_ref_philox4x32_10(c, k, o)
    return np.array(list(o), dtype=np.uint32)


def draw(seed, index, tag, level, iteration, chain) -> np.ndarray:
    o = (C.c_uint32 * 4)()
    lib().nuts_ref_draw(int(seed), int(index), int(tag), int(level), int(iteration), int(chain), o)
    return np.array(list(o), dtype=np.uint32)


def uniform(a, b) -> float:
    return float(lib().nuts_ref_uniform(int(a), int(b)))


def normal_pair(words) -> tuple[float, float]:
    w = (C.c_uint32 * 4)(*[int(x) for x in words])
    z = (C.c_double * 2)()
    lib().nuts_ref_normal_pair(w, z)
    return float(z[0]), float(z[1])


def logaddexp(a, b) -> float:
    return float(lib().nuts_ref_logaddexp(float(a), float(b)))


class Target:
    """Host-side description of a target for the oracle.  `dtype` is np.float32/64."""

    def __init__(self, kind, dim, dtype=np.float64, precision=None, scales=None, X=None, y=None, prior_scale=1.0):
        self.kind = int(kind)
        self.dim = int(dim)
        self.np_dtype = np.dtype(dtype)
        assert self.np_dtype in (np.dtype(np.float32), np.dtype(np.float64))
        self.dtype = F64 if self.np_dtype == np.dtype(np.float64) else F32
        cv = lambda a: None if a is None else np.ascontiguousarray(np.asarray(a), dtype=self.np_dtype)
        self.precision, self.scales, self.X, self.y = cv(precision), cv(scales), cv(X), cv(y)
        self.n_data = 0 if self.X is None else int(self.X.shape[0])
        self.prior_scale = float(prior_scale)

    def _args(self):
        p = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
        return [self.dtype, self.kind, self.dim, p(self.precision), p(self.scales), p(self.X), p(self.y),
                self.n_data, self.prior_scale]


def logp_grad(t: Target, theta):
    th = np.ascontiguousarray(theta, dtype=t.np_dtype)
    g = np.empty(t.dim, dtype=t.np_dtype)
    lp = C.c_double()
    rc = lib().nuts_ref_logp_grad(*t._args(), th.ctypes.data_as(C.c_void_p), g.ctypes.data_as(C.c_void_p), C.byref(lp))
    if rc:
        raise ValueError("nuts_ref_logp_grad: bad argument")
    return lp.value, g


def leapfrog(t: Target, theta, r, h, n_steps=1):
    th = np.array(theta, dtype=t.np_dtype, copy=True)
    rr = np.array(r, dtype=t.np_dtype, copy=True)
    lp = C.c_double()
    rc = lib().nuts_ref_leapfrog(*t._args(), th.ctypes.data_as(C.c_void_p), rr.ctypes.data_as(C.c_void_p),
                                 float(h), int(n_steps), C.byref(lp))
    if rc:
        raise ValueError("nuts_ref_leapfrog: bad argument")
    return th, rr, lp.value


def uturn_ok(tm, rm, tp, rp, dtype=np.float64) -> bool:
    a = [np.ascontiguousarray(x, dtype=dtype) for x in (tm, rm, tp, rp)]
    code = F64 if np.dtype(dtype) == np.dtype(np.float64) else F32
    return bool(lib().nuts_ref_uturn_ok(code, a[0].size, *[x.ctypes.data_as(C.c_void_p) for x in a]))


def sample(t: Target, n_chains, n_iters, step_size, max_tree_depth, seed, chain_ids=None, init_states=None,
           n_threads=1, want_margin=False, leaf_steps=1, sampler=MULTINOMIAL):
    """Returns (states [n_iters, n_chains, dim], tree_depths, n_leapfrog[, margin])."""
    n_chains, n_iters = int(n_chains), int(n_iters)
    states = np.empty((n_iters, n_chains, t.dim), dtype=t.np_dtype)
    depths = np.empty((n_iters, n_chains), dtype=np.int32)
    nleap = np.empty((n_iters, n_chains), dtype=np.int32)
    margin = np.empty((n_iters, n_chains), dtype=np.float64) if want_margin else None
    ids = None
    if chain_ids is not None:
        ids = np.ascontiguousarray(chain_ids, dtype=np.int64)
        assert ids.shape == (n_chains,)
    init = None
    if init_states is not None:
        init = np.ascontiguousarray(init_states, dtype=t.np_dtype)
        assert init.shape == (n_chains, t.dim)
    p = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
    rc = lib().nuts_ref_sample_k(*t._args(), n_chains, p(ids), p(init), n_iters, float(step_size),
                                 int(max_tree_depth), int(leaf_steps), int(sampler), int(seed), p(states), p(depths), p(nleap),
                                 p(margin), int(n_threads))
    if rc:
        raise ValueError("nuts_ref_sample: bad argument")
    return (states, depths, nleap, margin) if want_margin else (states, depths, nleap)
