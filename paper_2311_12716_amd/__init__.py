"""MI355X-native batched maze environment (student step, egocentric render,
teacher editor env, GAE) behind a C-ABI HIP library.

``paper_2311_12716_amd.binding`` holds the ctypes binding of the library;
``paper_2311_12716_amd.workloads`` the seeded synthetic input generators.
The binding is imported lazily so that the generators can be used on a machine
without the built library.
"""
__all__ = ["binding", "workloads"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
