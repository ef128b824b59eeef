"""MI355X-native GradiVeQ slice-wise linear PCA gradient codec (HIP kernels behind a C ABI)."""
from .configs import WORKLOADS, Workload  # noqa: F401
