"""MI355X-native HiRE decode-step hot path (HiRE-FFN, HiRE-Softmax, top-k select).

Sub-modules are imported on demand so that the input generators can be used
without the GPU library:

  inputs  seeded synthetic tensors (no method arithmetic)
  hire    ctypes binding of the C-ABI library libhire.so (fails loudly if it is not built)
  cost    parameter-byte accounting used by the benchmark
  hiprt   event timing on the loaded HIP runtime
  build   compiles the HIP sources for gfx950
"""
import importlib

_SUBMODULES = ("inputs", "hire", "hiprt", "cost", "build")


def __getattr__(name):
    if name in _SUBMODULES:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
