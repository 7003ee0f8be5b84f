"""MI355X-native data-parallel hot path of Synkhronos (arXiv 1710.04162).

The product is libsynk.so (HIP kernels for gfx950 behind the C ABI declared in
include/synk.h).  `paper_1710_04162_amd.binding` is its thin Python binding:
the functions have the C names and only marshal arguments (torch tensors ->
device pointers, the current torch stream -> hipStream_t).  There is no CPU
fallback: importing the binding without the built library raises.
`paper_1710_04162_amd.build` compiles the library in-tree.
"""


def __getattr__(name):
    # binding is loaded on first use so that `-m paper_1710_04162_amd.build`
    # works before the library exists
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
