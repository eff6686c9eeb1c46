"""MI355X-native gossiping-SGD aggregation step (arXiv 1611.04581).

`paper_1611_04581_amd.gsgd` is the thin ctypes binding over libgsgd.so (hand-written
HIP kernels for gfx950); `paper_1611_04581_amd.workloads` names the benchmark
shapes and draws seeded inputs.  The binding is imported lazily so that the
shape tables can be used without the GPU library being loaded.
"""
import importlib

__all__ = ["gsgd", "workloads"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
