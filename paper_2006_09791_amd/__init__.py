"""MI355X (gfx950) grouped-convolution library: Python side.

`workloads` holds seeded input recipes; `binding` marshals arguments to the
C-ABI library libgspc.so, which does all the work in HIP kernels.
"""
__all__ = ["workloads", "binding"]
