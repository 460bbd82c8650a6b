"""The C-ABI library: it loads, exports every symbol the header declares, and rejects bad arguments
on the host before touching a device.  No compute happens here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1910_11141_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "nuts.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nuts_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layouts_match_the_header():
    assert C.sizeof(B.nuts_target_desc) == 64
    assert C.sizeof(B.nuts_stats) == 72
    assert C.sizeof(B.nuts_sample_options) == 32


def test_create_target_rejects_bad_descriptors():
    lib = B.lib()
    out = C.c_void_p()
    assert lib.nuts_create_target(None, C.byref(out)) == B.NUTS_E_INVALID_ARG
    d = B.nuts_target_desc(0, 1, 2, None, None, None, None, 0, 1.0)
    assert lib.nuts_create_target(C.byref(d), None) == B.NUTS_E_INVALID_ARG
    for kw in [dict(kind=9), dict(kind=-1), dict(dtype=2), dict(dim=0), dict(kind=1), dict(kind=2), dict(kind=3)]:
        d = B.nuts_target_desc(0, 1, 2, None, None, None, None, 0, 1.0)
        for k, v in kw.items():
            setattr(d, k, v)
        assert lib.nuts_create_target(C.byref(d), C.byref(out)) == B.NUTS_E_INVALID_ARG, kw
        assert B.nuts_last_error()
    X = np.ones((3, 2)); y = np.array([0.0, 1.0, 2.0])
    with pytest.raises(B.NutsError) as e:
        B.Target(B.NUTS_TARGET_LOGISTIC_REGRESSION, 2, X=X, y=y)
    assert e.value.code == B.NUTS_E_INVALID_ARG and "y[2]" in str(e.value)
    with pytest.raises(B.NutsError):
        B.Target(B.NUTS_TARGET_LOGISTIC_REGRESSION, 2, X=X, y=np.zeros(3), prior_scale=0.0)
    with pytest.raises(B.NutsError):
        B.Target(B.NUTS_TARGET_GAUSS_DIAG, 2, scales=np.array([1.0, -1.0]))
    with pytest.raises(B.NutsError):
        B.Target(B.NUTS_TARGET_GAUSS_DENSE_PRECISION, 2, precision=np.array([[1.0, np.nan], [0.0, 1.0]]))


def test_sample_rejects_bad_arguments_before_touching_the_device():
    lib = B.lib()
    t = B.Target(B.NUTS_TARGET_STD_NORMAL, 2)     # needs no device
    good = dict(n_chains=4, n_iters=3, step_size=0.5, depth=6)
    for bad in [dict(n_chains=0), dict(n_iters=0), dict(step_size=0.0), dict(step_size=-1.0),
                dict(step_size=float("nan")), dict(step_size=float("inf")), dict(depth=0), dict(depth=21)]:
        a = dict(good); a.update(bad)
        rc = lib.nuts_sample(t.handle, a["n_chains"], a["n_iters"], a["step_size"], a["depth"], 1, None, None, None)
        assert rc == B.NUTS_E_INVALID_ARG, bad
    assert lib.nuts_sample(None, 4, 3, 0.5, 6, 1, None, None, None) == B.NUTS_E_INVALID_ARG
    opt = B.nuts_sample_options(None, 0, 7, 0)
    assert lib.nuts_sample_ex(t.handle, 4, 3, 0.5, 6, 1, C.byref(opt), None, None, None) == B.NUTS_E_INVALID_ARG
    opt = B.nuts_sample_options(None, -1, 0, 0)
    assert lib.nuts_sample_ex(t.handle, 4, 3, 0.5, 6, 1, C.byref(opt), None, None, None) == B.NUTS_E_INVALID_ARG
    opt = B.nuts_sample_options(None, 0, B.NUTS_VARIANT_TILE, 0)
    assert lib.nuts_sample_ex(t.handle, 4, 3, 0.5, 6, 1, C.byref(opt), None, None, None) == B.NUTS_E_UNSUPPORTED
    big = B.Target(B.NUTS_TARGET_STD_NORMAL, 5000)
    opt = B.nuts_sample_options(None, 0, B.NUTS_VARIANT_ELEM, 0)
    assert lib.nuts_sample_ex(big.handle, 4, 3, 0.5, 6, 1, C.byref(opt), None, None, None) == B.NUTS_E_UNSUPPORTED
    s = B.nuts_stats()
    assert lib.nuts_get_stats(t.handle, C.byref(s)) == B.NUTS_E_INVALID_ARG   # nothing has run
    assert lib.nuts_get_stats(None, C.byref(s)) == B.NUTS_E_INVALID_ARG
    assert lib.nuts_destroy_target(None) == B.NUTS_OK


def test_no_cpu_fallback_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    t = B.Target(B.NUTS_TARGET_STD_NORMAL, 2)
    with pytest.raises(B.NutsError) as e:
        B.nuts_sample(t, 4, 3, 0.5, 6, 1)
    assert e.value.code == B.NUTS_E_DEVICE
    with pytest.raises(B.NutsError) as e:
        B.Target(B.NUTS_TARGET_GAUSS_DIAG, 2, scales=np.ones(2))
    assert e.value.code == B.NUTS_E_DEVICE


def test_product_package_does_not_reference_the_oracle():
    pkg = os.path.join(ROOT, "paper_1910_11141_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "nuts_ref" not in text, os.path.join(dirpath, f)
                assert not re.search(r"^\s*(from|import)\s+oracle", text, flags=re.M), os.path.join(dirpath, f)
                assert "oracle/" not in text, os.path.join(dirpath, f)
