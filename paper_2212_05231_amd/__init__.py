"""MI355X-native hot path of NeuS2 (arXiv 2212.05231): one training step over a
batch of ray samples, behind a C-ABI library of hand-written HIP kernels.

Importing this package loads nothing native; `binding.lib()` loads the shared
library on first use and raises if it has not been built.
"""
