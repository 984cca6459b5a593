"""MI355X-native forward pass of NanoQuant's low-rank binary linear layer.

y = s_out (.) ( U . ( V^T . ( s_in (.) x ) ) )      (Section 3.1, Eq. 1)

The computation lives in a C-ABI shared library built from ``csrc/`` (HIP,
gfx950); ``binding`` is a thin ctypes layer over it and ``synth`` draws the
seeded synthetic workloads.  Nothing here falls back to a CPU implementation:
using the binding without the built library raises.
"""
__all__ = ["binding", "synth"]
