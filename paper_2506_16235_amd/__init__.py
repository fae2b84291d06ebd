"""NetSenseML gradient data-reduction hot path on MI355X (gfx950).

`paper_2506_16235_amd.binding` is a ctypes wrapper around the C-ABI library
`libnsml.so` (hand-written HIP kernels; see include/nsml.h).  Importing the
package itself is cheap; the library is loaded on first use and the import of
`binding` fails loudly if it has not been built.  There is no CPU fallback.
"""
__all__ = ["binding", "workloads"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
