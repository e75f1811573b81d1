"""pdelta: 1-bit per-axis weight-delta linear layers on MI355X (gfx950).

The work is done by hand-written HIP kernels behind a C-ABI shared library
(``include/pdelta.h``); ``binding`` marshals torch tensors to its pointers and nothing else.
``synth`` draws the seeded synthetic inputs used by tests and benches.  Importing the package
does not load the library; the first call does, and raises if it has not been built.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
