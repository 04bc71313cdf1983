"""MI355X (gfx950) implementation of the batched per-agent recurrent Q-network
used by the worker decision step (Alg. 2) and the learner TD step (Alg. 3).

`workloads` holds the seeded input generators; `binding` is the thin ctypes
layer over the C-ABI library built from csrc/.  Nothing here falls back to a
CPU implementation: calling a compute entry point without the built HIP
library raises.
"""
__all__ = ["workloads", "binding"]
