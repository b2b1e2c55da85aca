"""MI355X-native Sparsely-Gated Mixture-of-Experts layer (hot path of arXiv 1701.06538).

`paper_1701_06538_amd.api` is a thin ctypes binding over the C ABI declared in include/moe.h;
every step of the layer runs in the HIP kernels of libmoe_hip.so.  There is no CPU fallback:
importing `api` fails loudly when the library has not been built.
"""
__all__ = ["api", "build"]
