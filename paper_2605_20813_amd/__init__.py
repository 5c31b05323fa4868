"""MI355X-native PulseCol attention hot path (column-sparse attention for diffusion LLMs).

``paper_2605_20813_amd.pulsecol`` is the thin ctypes binding over the C-ABI
library built from ``csrc/``; ``paper_2605_20813_amd.workloads`` draws the
seeded synthetic inputs; ``paper_2605_20813_amd.schedule`` drives the refresh
schedule over a stack of layers.  Importing the package loads neither torch nor the
shared library; the binding does so on first use and raises if the library
has not been built.
"""

__all__ = ["pulsecol", "workloads", "schedule"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
