"""libburstattn: the per-device compute step of BurstAttention on MI355X.

`binding` (loaded on first attribute access) wraps the C-ABI library;
`workloads` holds the seeded synthetic inputs.  Importing the package alone
touches neither the GPU nor the shared library.
"""
import importlib

__all__ = ["binding", "workloads", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
