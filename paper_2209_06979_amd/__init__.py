"""MI355X-native quantized vector-sparse SpMM / SDDMM / sparse attention (gfx950 HIP).

``binding`` wraps the C ABI declared in include/magicube.h; ``workloads`` draws the
seeded synthetic inputs; ``build`` compiles the shared library in-tree.
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    # the binding loads libmagicube.so at import and fails loudly when it is missing
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
