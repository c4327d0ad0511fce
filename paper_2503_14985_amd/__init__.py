"""MI355X-native tile kernels behind a C ABI: ``mlt_gemm`` and ``mlt_mha_fwd``.

The package holds the HIP sources (``csrc/``), the ctypes binding (``binding``) and the seeded
synthetic input generators (``inputs``). Nothing is imported eagerly, so ``inputs`` can be used
on a machine without the built GPU library; every compute entry point raises if the library is
missing.
"""

__all__ = ["binding", "inputs"]
