"""MI355X-native fused dequantise-and-multiply GEMM for fine-grained weight-only quantisation.

The work is done by hand-written HIP kernels behind a C ABI (``include/fq.h``,
``libfq.so``); ``paper_2308_09723_amd.fq`` is the thin binding.  Nothing here
falls back to a CPU or PyTorch implementation: if the library is missing the
binding raises.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "fq"]


def __getattr__(name):
    if name == "fq":
        import importlib

        return importlib.import_module(".fq", __name__)
    raise AttributeError(name)
