"""Lock-step NUTS on MI355X: Python face of the C-ABI library (see include/nuts.h)."""
import importlib

from . import workloads  # noqa: F401  (pure numpy: safe without the HIP library)


def __getattr__(name):
    # The binding is loaded on first use so that `workloads` stays importable on a
    # machine where the library has not been built; using the sampler without the
    # library raises (there is no CPU path).
    if name.startswith("__"):
        raise AttributeError(name)
    binding = importlib.import_module(__name__ + ".binding")
    return getattr(binding, name)
