"""PowerGossip hot path for MI355X (gfx950): C-ABI HIP library + thin Python binding.

``workloads`` holds the seeded synthetic inputs; ``binding`` (imported lazily, it
needs the built ``libpowergossip.so``) mirrors the C entry points one to one.
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
