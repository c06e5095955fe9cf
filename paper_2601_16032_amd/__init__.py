"""Sawtooth Wavefront Reordering attention forward for MI355X (gfx950).

The product is the C-ABI library built from csrc/ (hand-written HIP); `binding` marshals
arguments to it.  Nothing here falls back to a CPU or PyTorch implementation: if the library is
missing, calls raise.
"""
