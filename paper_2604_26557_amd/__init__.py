"""MI355X-native hot path of dual-path KV-cache offloading.

The GPU library (extent planner, pack/unpack kernels, chunk pipeline, split-K decode
attention) sits behind a C ABI; `binding` marshals arguments to it and nothing else.
`workloads` holds the seeded synthetic inputs and imports neither the binding nor torch
device state, so importing this package never loads the native library.
"""

__all__ = ["binding", "workloads", "build"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
