"""Thin ctypes binding of the C ABI in include/nuts.h.

Argument marshalling only: every step of the sampler runs in the HIP library.
PyTorch supplies device memory (output tensors) and the stream.  If the shared
library is missing the import fails; nothing here computes on the CPU.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnuts_hip.so")

NUTS_OK, NUTS_E_INVALID_ARG, NUTS_E_ALLOC, NUTS_E_DEVICE, NUTS_E_UNSUPPORTED = 0, -1, -2, -3, -4
NUTS_F32, NUTS_F64 = 0, 1
NUTS_TARGET_STD_NORMAL, NUTS_TARGET_GAUSS_DENSE_PRECISION, NUTS_TARGET_GAUSS_DIAG, NUTS_TARGET_LOGISTIC_REGRESSION = 0, 1, 2, 3
NUTS_VARIANT_AUTO, NUTS_VARIANT_WAVE, NUTS_VARIANT_TILE, NUTS_VARIANT_ELEM, NUTS_VARIANT_GRID = 0, 1, 2, 3, 4
NUTS_VARIANT_DENSE, NUTS_VARIANT_QUAD = 5, 6
NUTS_SCHEDULE_FREE, NUTS_SCHEDULE_TRAJECTORY = 0, 1
NUTS_SAMPLER_MULTINOMIAL, NUTS_SAMPLER_SLICE = 0, 1

EXPORTS = ("nuts_create_target", "nuts_destroy_target", "nuts_sample", "nuts_sample_ex", "nuts_get_stats",
           "nuts_sample_static", "nuts_set_stream", "nuts_tile_pack", "nuts_last_error")
NUTS_STATIC_SCRATCH_BYTES = 64 << 20


class nuts_target_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("dim", C.c_int64), ("precision", C.c_void_p),
                ("scales", C.c_void_p), ("X", C.c_void_p), ("y", C.c_void_p), ("n_data", C.c_int64),
                ("prior_scale", C.c_double)]


class nuts_stats(C.Structure):
    _fields_ = [("leaf_slots_issued", C.c_uint64), ("leaf_slots_useful", C.c_uint64),
                ("extra_grad_evals", C.c_uint64), ("rounds", C.c_uint64), ("kernel_ms", C.c_double),
                ("phase_ticks", C.c_uint64 * 3), ("variant", C.c_int32), ("grid_blocks", C.c_int32)]


class nuts_sample_options(C.Structure):
    _fields_ = [("init_states", C.c_void_p), ("first_chain", C.c_int64), ("variant", C.c_int32),
                ("leaf_steps", C.c_int32), ("schedule", C.c_int32), ("sampler", C.c_int32)]


class NutsError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"nuts error {code}: {message}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime; it has to be in the process before this library is, so that both
        # resolve the runtime's soname to the same copy (two copies do not see each other's device state)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.nuts_create_target.argtypes = [C.POINTER(nuts_target_desc), C.POINTER(C.c_void_p)]
        L.nuts_destroy_target.argtypes = [C.c_void_p]
        common = [C.c_void_p, C.c_int64, C.c_int64, C.c_double, C.c_int32, C.c_uint64]
        L.nuts_sample.argtypes = common + [C.c_void_p, C.c_void_p, C.c_void_p]
        L.nuts_sample_ex.argtypes = common + [C.POINTER(nuts_sample_options), C.c_void_p, C.c_void_p, C.c_void_p]
        L.nuts_sample_static.argtypes = L.nuts_sample_ex.argtypes
        L.nuts_get_stats.argtypes = [C.c_void_p, C.POINTER(nuts_stats)]
        L.nuts_set_stream.argtypes = [C.c_void_p]
        L.nuts_last_error.argtypes = []
        L.nuts_last_error.restype = C.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class nuts_tile_layout(C.Structure):
    _fields_ = [("ks1", C.c_int32), ("mt", C.c_int32), ("n_tiles", C.c_int32), ("n_alloc_tiles", C.c_int32),
                ("const_col", C.c_int32), ("reserved", C.c_int32), ("const_val", C.c_double), ("n_pad", C.c_int64),
                ("operand_doubles", C.c_int64)]


def nuts_tile_pack(X, y):
    """Host only: the tile variant's operand stream for a binary64 logistic-regression data set (numpy arrays X n x d,
    y n).  Returns (layout as a dict, the stream as a float64 array)."""
    import numpy as np
    X = np.ascontiguousarray(X, dtype=np.float64)
    y = np.ascontiguousarray(y, dtype=np.float64)
    n, d = X.shape
    lay = nuts_tile_layout()
    px, py = X.ctypes.data_as(C.c_void_p), y.ctypes.data_as(C.c_void_p)
    _check(lib().nuts_tile_pack(px, py, C.c_int64(n), C.c_int64(d), C.byref(lay), None, C.c_int64(0)))
    out = np.empty(lay.operand_doubles, dtype=np.float64)
    _check(lib().nuts_tile_pack(px, py, C.c_int64(n), C.c_int64(d), C.byref(lay), out.ctypes.data_as(C.c_void_p),
                                C.c_int64(out.size)))
    return {f: getattr(lay, f) for f, _ in nuts_tile_layout._fields_ if f != "reserved"}, out


def nuts_last_error() -> str:
    return lib().nuts_last_error().decode()


def _check(rc: int):
    if rc != NUTS_OK:
        raise NutsError(rc, nuts_last_error())


def _np_dtype(dtype_code: int):
    return np.float64 if dtype_code == NUTS_F64 else np.float32


def nuts_create_target(kind: int, dim: int, dtype=np.float64, *, precision=None, scales=None, X=None, y=None,
                       prior_scale: float = 1.0) -> "Target":
    return Target(kind, dim, dtype, precision=precision, scales=scales, X=X, y=y, prior_scale=prior_scale)


class Target:
    """Owns a nuts_target handle.  Host arrays are copied by the library."""

    def __init__(self, kind, dim, dtype=np.float64, *, precision=None, scales=None, X=None, y=None, prior_scale=1.0):
        npdt = np.dtype(dtype)
        if npdt not in (np.dtype(np.float32), np.dtype(np.float64)):
            raise ValueError("dtype must be float32 or float64")
        self.np_dtype = npdt
        self.dtype = NUTS_F64 if npdt == np.dtype(np.float64) else NUTS_F32
        self.kind, self.dim = int(kind), int(dim)
        cv = lambda a: None if a is None else np.ascontiguousarray(np.asarray(a), dtype=npdt)
        arrs = dict(precision=cv(precision), scales=cv(scales), X=cv(X), y=cv(y))
        ptr = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
        n_data = 0 if arrs["X"] is None else int(arrs["X"].shape[0])
        if arrs["X"] is not None and (arrs["X"].ndim != 2 or arrs["X"].shape[1] != self.dim or arrs["y"] is None
                                      or arrs["y"].shape != (n_data,)):
            raise ValueError("X must be [n_data, dim] and y [n_data]")
        if arrs["precision"] is not None and arrs["precision"].shape != (self.dim, self.dim):
            raise ValueError("precision must be [dim, dim]")
        if arrs["scales"] is not None and arrs["scales"].shape != (self.dim,):
            raise ValueError("scales must be [dim]")
        desc = nuts_target_desc(self.kind, self.dtype, self.dim, ptr(arrs["precision"]), ptr(arrs["scales"]),
                                ptr(arrs["X"]), ptr(arrs["y"]), n_data, float(prior_scale))
        handle = C.c_void_p()
        _check(lib().nuts_create_target(C.byref(desc), C.byref(handle)))
        self.handle = handle
        self.n_data = n_data

    def close(self):
        if getattr(self, "handle", None):
            lib().nuts_destroy_target(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def nuts_set_stream(stream) -> None:
    """`stream`: a torch.cuda.Stream, a raw hipStream_t integer, or None for the null stream."""
    raw = 0 if stream is None else int(getattr(stream, "cuda_stream", stream))
    _check(lib().nuts_set_stream(C.c_void_p(raw)))


def nuts_sample(target: Target, n_chains: int, n_iters: int, step_size: float, max_tree_depth: int, seed: int, *,
                init_states=None, first_chain: int = 0, variant: int = NUTS_VARIANT_AUTO, out=None,
                want_states: bool = True, leaf_steps: int = 1, schedule: int = NUTS_SCHEDULE_FREE,
                sampler: int = NUTS_SAMPLER_MULTINOMIAL, static_scratch: bool = False):
    """Enqueue a sampling run; returns (states, tree_depths, n_leapfrog) as CUDA tensors.
    The caller synchronises (e.g. torch.cuda.synchronize()) before reading them."""
    import torch

    tdt = torch.float64 if target.dtype == NUTS_F64 else torch.float32
    dev = torch.device("cuda", torch.cuda.current_device()) if torch.cuda.is_available() else None
    if dev is None:
        # No device: hand the library null outputs so that it reports the device error itself.
        states = depths = nleap = None
    elif out is not None:
        states, depths, nleap = out
        for t, shape, dt in ((states, (n_iters, n_chains, target.dim), tdt), (depths, (n_iters, n_chains), torch.int32),
                             (nleap, (n_iters, n_chains), torch.int32)):
            # the library writes through raw pointers: a wrong buffer would be an out-of-bounds device write
            if t is not None and not (t.is_cuda and t.device == dev and t.dtype == dt and t.is_contiguous()
                                      and tuple(t.shape) == shape):
                raise ValueError(f"out tensor must be a contiguous {dt} CUDA tensor of shape {shape} on {dev}")
    else:
        states = torch.empty((n_iters, n_chains, target.dim), dtype=tdt, device=dev) if want_states else None
        depths = torch.empty((n_iters, n_chains), dtype=torch.int32, device=dev)
        nleap = torch.empty((n_iters, n_chains), dtype=torch.int32, device=dev)
    opt = nuts_sample_options(None, int(first_chain), int(variant), int(leaf_steps), int(schedule), int(sampler))
    if init_states is not None:
        assert init_states.is_cuda and init_states.dtype == tdt and init_states.is_contiguous()
        assert tuple(init_states.shape) == (n_chains, target.dim)
        opt.init_states = init_states.data_ptr()
    p = lambda t: None if t is None else C.c_void_p(t.data_ptr())
    entry = lib().nuts_sample_static if static_scratch else lib().nuts_sample_ex
    _check(entry(target.handle, int(n_chains), int(n_iters), float(step_size), int(max_tree_depth),
                                int(seed) & 0xFFFFFFFFFFFFFFFF, C.byref(opt), p(states), p(depths), p(nleap)))
    return states, depths, nleap


def nuts_get_stats(target: Target) -> dict:
    s = nuts_stats()
    _check(lib().nuts_get_stats(target.handle, C.byref(s)))
    d = {name: getattr(s, name) for name, _ in nuts_stats._fields_}
    d["phase_ticks"] = list(s.phase_ticks)
    d["occupancy"] = d["leaf_slots_useful"] / d["leaf_slots_issued"] if d["leaf_slots_issued"] else float("nan")
    return d
