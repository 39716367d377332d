"""MI355X-native batched 2D-convolution hot path of DLL (arxiv 1804.04512).

`workloads` (seeded synthetic inputs) is importable anywhere; `binding` loads the
HIP library and fails loudly when it has not been built.
"""
