"""MI355X-native compress / restore path of LC-Checkpoint (arXiv 2009.13003).

`lc` (the ctypes binding of the HIP library) is imported lazily so that the
input generators in `workloads` can be used without the library being built.
"""


def __getattr__(name):
    if name == "lc":
        import importlib
        return importlib.import_module(".lc", __name__)
    raise AttributeError(name)
