"""ReAttention per-layer attention hot path for AMD MI355X (gfx950).

`paper_2407_15176_amd.binding` is the thin ctypes front of the C-ABI library
libreattn.so (hand-written HIP kernels); `paper_2407_15176_amd.workloads` holds
the seeded synthetic input recipes.  Nothing here falls back to a CPU path.
"""
__all__ = ["binding", "workloads"]
