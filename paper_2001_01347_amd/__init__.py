"""MI355X-native ZipLine barrier search (ElasticBSP, arXiv 2001.01347).

``workloads`` draws the seeded synthetic inputs; ``zipline`` is the thin ctypes
binding over the HIP library built from ``csrc/``.  The binding loads the
library on first use and raises if it has not been built: there is no CPU
fallback.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "zipline"]


def __getattr__(name):
    if name == "zipline":
        import importlib
        return importlib.import_module(".zipline", __name__)
    raise AttributeError(name)
