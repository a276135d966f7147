"""MI355X-native forward pass of an APB layer (arXiv 2306.08960): C-ABI HIP library + thin binding.

`binding` wraps libapb.so (built in-tree by `build.py`); `synth` draws the seeded synthetic
layers used by tests and the benchmark.  There is no CPU implementation in this package.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
