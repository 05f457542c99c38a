"""MI355X-native conv-GLU + CTC training path (wav2letter++ acoustic-model hot path).

The product is ``libw2l.so`` (hand-written HIP for gfx950 behind a C ABI, see
``include/w2l.h``); this package is the thin binding that marshals torch device
tensors into it.  There is no CPU fallback: the first use of any entry point loads the
library and raises if it has not been built (``python -m paper_1812_07625_amd.build``).
The binding is resolved lazily so that the build module can be imported before the
library exists.
"""
import importlib

_binding = None


def _load_binding():
    global _binding
    if _binding is None:
        _binding = importlib.import_module(".binding", __name__)
    return _binding


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    if name in ("build", "binding"):
        return importlib.import_module("." + name, __name__)
    return getattr(_load_binding(), name)


def __dir__():
    return sorted(set(globals()) | set(dir(_load_binding())))
