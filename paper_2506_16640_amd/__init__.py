"""MI355X-native alpha-entmax / ASEntmax attention (forward + backward).

The compute path is the C-ABI library built from csrc/ (hand-written HIP for
gfx950); `binding` marshals torch device tensors into it.  `synth` only draws
seeded inputs.  Import `paper_2506_16640_amd.binding` to use the kernels: it
raises if the library has not been built.
"""
__all__ = ["binding", "synth"]
