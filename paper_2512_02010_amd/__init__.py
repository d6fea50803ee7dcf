"""Four Over Six (4/6) NVFP4 quantization for AMD MI355X (gfx950).

The product is the C-ABI library ``libnvfp4_46.so`` (``csrc/``, declared in
``include/nvfp4_46.h``); :mod:`.binding` marshals arguments to it and
:mod:`.workloads` draws the synthetic benchmark tensors.  Nothing here falls
back to a CPU implementation.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding", "build"]


def __getattr__(name):
    if name in ("binding", "build"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
