"""MI355X-native top-p selection + sparse decode attention (SpecAttn hot path).

`workloads` draws synthetic inputs and is importable anywhere.  The binding to
the HIP library (`paper_2510_27641_amd.binding`) is imported lazily so that
CPU-only code can use the input generators without a GPU.
"""

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
