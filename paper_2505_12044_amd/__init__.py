"""MI355X-native low-rank-bias attention (FlashBias, arxiv 2505.12044): HIP kernels behind
a C-ABI (include/flashbias.h) plus a thin ctypes binding.

Importing the package does not load the native library; the first call does, and it fails
loudly if the library has not been built (there is no CPU fallback)."""

__all__ = ["api", "autograd", "workloads"]
