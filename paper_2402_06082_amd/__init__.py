"""SubGen per-token decode step for MI355X (gfx950): HIP kernels behind a C-ABI library.

``binding`` exposes the C entry points one to one; ``workloads`` holds the
seeded synthetic input generators.  Importing the package does not load the
HIP library; the first call through ``binding`` does, and raises if it has
not been built.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
