"""MI355X-native batched evaluator of the Themis collective chunk scheduler
(arXiv 2110.04478): thin Python binding over the C ABI in include/themis.h.

`workloads` (numpy only) builds seeded scenario batches; `binding` marshals
torch device tensors into the C ABI.  Every step of the path runs in the HIP
kernels of libthemis_hip.so; there is no CPU fallback.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
