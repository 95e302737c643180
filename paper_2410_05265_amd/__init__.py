"""MI355X-native statically quantized W4A4 linear layer (PrefixQuant's inference hot path).

The product is libpq.so (HIP kernels behind the C ABI of include/pq.h); `binding` is the
thin ctypes layer over it and `synth` the seeded input generators.
"""

from . import synth  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
