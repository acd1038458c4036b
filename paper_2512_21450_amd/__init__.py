"""Shared-prefix grouped-query decode attention for GRPO-style rollouts on MI355X.

``workloads`` (seeded synthetic inputs) imports without the native library;
``binding`` loads the HIP library and raises if it has not been built.
"""
__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
