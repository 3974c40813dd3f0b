"""Measured device compute rate c_d for the scheduler's cost model.

The performance model prices a ring step at 16 * B * L_G * L_Gsrc * n_d * d_h / c_d (App. A.4, Eq. 11:
forward + backward + recomputation, no causal discount).  Instead of a data-sheet FLOP/s figure, c_d can be
the rate this library's kernels sustain in that same convention: one fully visible ring step (forward chunk
and backward chunk) is timed on the device and c_d = 16 * Lq * Lc * n_q * d_h / time.  All arithmetic runs in
the library's kernels; this module only allocates the buffers and reads HIP events.
"""
import torch

from . import hexi


def measure_c_d(head_dim=128, n_q_heads=8, n_kv_heads=2, lq=8192, lc=8192, device="cuda:0", reps=5, seed=0):
    """FLOP/s in the convention of Eq. 11 for a fully visible step of lq x lc tokens in bf16."""
    dev = torch.device(device)
    g = torch.Generator(device=dev).manual_seed(seed)
    rnd = lambda *shape: torch.randn(shape, device=dev, generator=g).to(torch.bfloat16)
    q, d_o = rnd(lq, n_q_heads, head_dim), rnd(lq, n_q_heads, head_dim)
    k, v = rnd(lc, n_kv_heads, head_dim), rnd(lc, n_kv_heads, head_dim)
    f32 = dict(dtype=torch.float32, device=dev)
    o, dq = torch.zeros((lq, n_q_heads, head_dim), **f32), torch.zeros((lq, n_q_heads, head_dim), **f32)
    lse, delta = torch.empty((n_q_heads, lq), **f32), torch.empty((n_q_heads, lq), **f32)
    dk, dv = torch.empty((lc, n_kv_heads, head_dim), **f32), torch.empty((lc, n_kv_heads, head_dim), **f32)
    desc = hexi.desc_for(q, k, head_dim ** -0.5)
    q_segs, kv_segs = [(lc, lq)], [(0, lc)]      # the shard lies after the chunk: every pair is visible

    def step():
        hexi.hexi_attn_fwd_chunk(desc, q_segs, kv_segs, q, k, v, o, lse)
        hexi.hexi_attn_bwd_chunk(desc, q_segs, kv_segs, q, k, v, o, d_o, lse, delta, dq, dk, dv, flags=hexi.HEXI_COMPUTE_DELTA)

    step()
    step()
    torch.cuda.synchronize(dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        step()
    e1.record()
    torch.cuda.synchronize(dev)
    seconds = e0.elapsed_time(e1) * 1e-3 / reps
    return 16.0 * lq * lc * n_q_heads * head_dim / seconds
