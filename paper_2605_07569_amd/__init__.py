"""MI355X-native chunked-ring causal attention: the per-device hot path of HexiSeq's CP-HP training.

`paper_2605_07569_amd.hexi` is the thin ctypes binding over the C-ABI library (HIP kernels for
gfx950); `paper_2605_07569_amd.workloads` builds the seeded synthetic shard configurations.
Nothing here falls back to a CPU implementation: using the binding without the built library raises.
"""
__all__ = ["hexi", "workloads"]
