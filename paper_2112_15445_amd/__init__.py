"""MI355X-native direct sparse convolution (HIP library + ctypes binding + workload generator)."""
from . import workloads  # noqa: F401  (pure numpy; no GPU code)

__all__ = ["workloads", "binding"]
