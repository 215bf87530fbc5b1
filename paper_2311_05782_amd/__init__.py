"""MI355X-native fault-injection campaigns on mixed-precision GEMM.

`paper_2311_05782_amd.fi` is the thin binding over the C-ABI library
(libfi_gfx950.so, built from csrc/); `paper_2311_05782_amd.workloads` draws
seeded synthetic inputs.  Nothing is loaded until it is used.
"""
__all__ = ["fi", "workloads"]
