"""MI355X-native batched PCGRL environment step: HIP kernels behind a C ABI, plus this binding."""
from . import workloads  # noqa: F401  (data only; safe without a GPU)

__all__ = ["workloads"]
