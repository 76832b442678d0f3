"""MI355X-native Bi-GCN forward pass (binary graph convolution): hand-written HIP kernels
behind a C ABI, with a thin ctypes binding.  Importing the package does not load the HIP
library; the first call into :mod:`paper_2210_13149_amd.binding` does, and fails loudly if
it has not been built."""

__version__ = "0.1.0"
