"""Focus-dLLM sparse-attention step for AMD MI355X: HIP kernels behind a C ABI, plus a ctypes binding."""
from . import binding  # noqa: F401

__all__ = ["binding"]
