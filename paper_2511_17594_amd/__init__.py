"""MI355X-native CSR SpMM / SDDMM / CSR-attention library (AutoSAGE hot path).

`paper_2511_17594_amd.binding` is the ctypes front end of libautosage.so (built by
`paper_2511_17594_amd.build.build_library()`); `paper_2511_17594_amd.workloads` holds the
seeded synthetic input generators.  Importing this package alone loads neither torch nor
the library; importing `.binding` fails loudly when the library has not been built.
"""
__all__ = ["binding", "workloads", "build"]
