"""MI355X-native BP-Transformer graph self-attention (arXiv 1911.04070).

The compute path is a C-ABI HIP library (``include/bpt.h``); ``binding`` is the
thin ctypes layer over it and ``workloads`` holds the synthetic configurations.
"""
