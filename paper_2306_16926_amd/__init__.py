"""MI355X-native OSP synchronization step (2-stage gradient synchronization
with PGP importance and LGP correction).

`workloads` (seeded synthetic inputs) imports nothing else from this package.
`binding` loads the HIP library; it is imported on first use so that the
workload tables stay usable where the library is not built.
"""

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
