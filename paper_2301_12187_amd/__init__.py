"""MI355X-native two-stage dynamic program for latency-aware depth compression.

`inputs` draws seeded synthetic tables (numpy only).  `api` is the thin
binding over the C-ABI library libdpc.so (hand-written HIP for gfx950); it is
imported lazily so that the input generators stay usable on a machine
without the built library, while any call into the solver without it fails
loudly.
"""
from . import inputs  # noqa: F401


def __getattr__(name):
    if name == "api":
        import importlib
        return importlib.import_module(".api", __name__)
    raise AttributeError(name)
