"""MI355X-native measurement-and-recovery path: sketch, structured sparse
recovery, block-sparse SwiGLU FFN, head-pruned decode attention and joint
token/channel selection, as hand-written HIP kernels behind a C ABI.

`paper_2604_14156_amd.binding` is the ctypes layer over the shared library;
`paper_2604_14156_amd.workloads` draws the seeded synthetic inputs.
"""
__all__ = ["binding", "workloads", "buildlib"]
