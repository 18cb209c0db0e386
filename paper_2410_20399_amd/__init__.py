"""MI355X-native fused exact softmax attention (forward and backward) behind a C ABI.

``from paper_2410_20399_amd import attn`` loads the HIP library lazily; importing
the package itself touches neither the GPU nor the shared library.
"""
__all__ = ["attn", "workloads"]
