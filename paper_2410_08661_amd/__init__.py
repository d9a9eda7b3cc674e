"""MI355X-native fused mixed-precision linear layer of QEFT (arxiv 2410.08661).

`binding` (loaded on first use) holds the ctypes binding of libqeft.so, the C-ABI
library declared in include/qeft.h; `synth` the seeded synthetic inputs; `build` the
hipcc build.  There is no CPU or PyTorch fallback for any operation.
"""
import importlib

__all__ = ["binding", "synth", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
