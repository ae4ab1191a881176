"""MI355X-native XNOR-Net binary convolution forward pass (HIP kernels behind a C ABI).

``binding`` loads the in-tree HIP library and fails if it has not been built; ``workloads`` holds
the benchmark layer shapes and seeded input recipes and needs no GPU.
"""
__all__ = ["binding", "workloads", "build"]
