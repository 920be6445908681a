"""MEFT sparse-adapter layer (router -> top-e blocks -> key scores -> top-k neurons ->
weighted value sum, and its sparse backward) for AMD MI355X (gfx950).

`synth` generates seeded inputs; `binding` loads the HIP library through its C ABI.
The binding is imported lazily so that the input generator is usable on machines
where the library has not been built.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(__name__ + ".binding")
    raise AttributeError(name)
