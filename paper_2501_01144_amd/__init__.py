"""DialectFP4 (BlockDialect) hot path for AMD MI355X: HIP kernels behind a C ABI.

`paper_2501_01144_amd.dfp4` is the ctypes binding of libdfp4.so (argument
marshalling only); `paper_2501_01144_amd.synth` holds seeded input recipes.
Importing this package loads nothing: the library is loaded on first use and
the binding raises if it has not been built.
"""
__all__ = ["dfp4", "synth"]
