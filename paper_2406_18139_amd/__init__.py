"""MI355X-native LOOK-M prefill-time KV-cache compression (HIP kernels behind a C ABI).

``lookm`` holds the ctypes binding to ``liblookm.so``; ``workloads`` the seeded synthetic
inputs.  The shared library is loaded on first use and there is no CPU fallback: calling
the path without the built library or without a GPU raises.
"""
__all__ = ["lookm", "workloads"]
