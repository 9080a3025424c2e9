"""Wave-index decode attention and segmented k-means index build for MI355X.

The compute path is a C-ABI shared library of hand-written HIP kernels
(`csrc/`, declared in `include/wave.h`); `binding` marshals torch tensors into
it.  `synth` generates seeded inputs and has no dependency on the library.
Nothing here falls back to a CPU implementation: using the binding without the
built library raises.
"""
__all__ = ["binding", "synth"]
