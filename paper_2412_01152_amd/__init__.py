"""DiLoCo outer-synchronisation kernels for AMD MI355X (gfx950).

The product is the C-ABI library built from csrc/ (see include/diloco_mi355.h); `binding` is the
thin ctypes layer over it and `synth` makes seeded synthetic inputs.  Nothing here falls back to a
CPU path: loading the binding without the built library raises.
"""
__all__ = ["binding", "synth"]
