"""MI355X-native sparse convolution (kernel maps + gather/matmul/scatter) behind a C ABI.

``paper_2204_10319_amd.binding`` is the thin ctypes layer over ``libts.so``;
``paper_2204_10319_amd.build`` compiles the library with hipcc.  Importing this package
does not load the library; the first call into the binding does, and fails loudly when
the shared object is missing.
"""

__all__ = ["binding", "build"]
