"""MI355X-native densify of assumed-sparse gradients (arXiv 1905.04035).

`binding` is the ctypes front end of the C-ABI library built from `csrc/`;
`workloads` draws seeded synthetic inputs; `build` compiles the library.
The binding is imported on first use so that `workloads` stays importable on a
machine where the library has not been built.
"""
import importlib

__all__ = ["binding", "workloads", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
