"""Cached embedding-bag training path (pooled lookup + sparse backward with
row-wise Adagrad through a set-associative LRU cache in HBM) for MI355X.

The HIP library binding lives in :mod:`paper_2305_01515_amd.tbe` and is loaded
on first attribute access, so that :mod:`paper_2305_01515_amd.synth` (seeded
input generators, no arithmetic of the method) can be imported on its own.
"""

__all__ = ["tbe", "synth"]


def __getattr__(name):
    if name in ("tbe", "synth"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
