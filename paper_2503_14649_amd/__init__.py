"""MI355X-native IVF-PQ and flat vector retrieval behind a C ABI (see include/rago.h).

`paper_2503_14649_amd.binding` is the ctypes binding; it is imported lazily so that tooling which
only needs the build script does not require a built library.
"""


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
