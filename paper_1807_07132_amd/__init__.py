"""MI355X-native local Newton-CG x-update of Newton-ADMM (softmax regression).

`nadmm`      ctypes binding of the C-ABI library (HIP kernels for gfx950)
`workloads`  seeded synthetic inputs shaped like the paper's data sets
"""
__all__ = ["nadmm", "workloads"]
