"""KVReviver decode hot path for AMD MI355X: HIP kernels behind a C ABI
(include/kvr.h, paper_2512_17917_amd/csrc) and their ctypes binding.

    from paper_2512_17917_amd import binding as kvr

`binding` loads paper_2512_17917_amd/libkvr.so on first use and raises if it
has not been built (python -m paper_2512_17917_amd.build).
"""
__all__ = ["binding", "build"]
