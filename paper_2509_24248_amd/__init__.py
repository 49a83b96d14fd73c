"""SpecExit decode-round hot path for AMD MI355X: HIP kernels behind a C ABI.

`binding` (imported on first use) loads libspecexit.so and raises if it has not been
built; `build` compiles it.  Nothing here computes on the CPU."""
import importlib

__all__ = ["binding", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
