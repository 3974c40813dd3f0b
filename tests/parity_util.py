"""Shared helpers of the GPU parity tests: tolerances and oracle-side evaluation of a workload."""
import numpy as np
import torch

import oracle
from paper_2605_07569_amd import workloads as wl

# Per output tensor.  bf16 inputs: max-abs <= 2e-2 and relative L2 <= 5e-3.  fp32 inputs: relative
# L2 <= 1e-5 and max-abs <= 1e-5 * max(1, max|ref|).
TOL = {"bf16": dict(max_abs=2e-2, rel_l2=5e-3), "f32": dict(max_abs=1e-5, rel_l2=1e-5)}


def check(name, got, ref, dtype, log=None, abs_factor=1.0):
    """abs_factor widens the max-abs bound for intermediates that are sums of d products of an output
    (Delta = <dO, O> inherits up to sqrt(d) * |dO| times the per-element error allowed for O)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin), f"{name}: finiteness pattern differs"
    assert np.array_equal(got[~fin], ref[~fin]), f"{name}: infinities differ"
    g, r = got[fin], ref[fin]
    max_abs = float(np.max(np.abs(g - r))) if g.size else 0.0
    rel_l2 = float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300)) if g.size else 0.0
    tol = TOL[dtype]
    lim_abs = abs_factor * tol["max_abs"] * (max(1.0, float(np.max(np.abs(r)))) if (dtype == "f32" and r.size) else 1.0)
    msg = f"{name}: max_abs={max_abs:.3e} (<= {lim_abs:.1e})  rel_l2={rel_l2:.3e} (<= {tol['rel_l2']:.1e})"
    if log is not None:
        log.append(msg)
    print("   ", msg, flush=True)
    assert max_abs <= lim_abs and rel_l2 <= tol["rel_l2"], msg
    return max_abs, rel_l2


def to64(t):
    return t.to(torch.float64).numpy()


def oracle_full(w, inputs, q_rows=None):
    """Exact results for the workload's shard (optionally a subset of its packed rows): o, lse, dq for
    those rows; dk, dv over the WHOLE global key range from those rows only."""
    q_pos = wl.seg_positions(w.q_segs).numpy()
    q, d_o = to64(inputs["q"]), to64(inputs["d_o"])
    if q_rows is not None:
        q, d_o, q_pos = q[q_rows], d_o[q_rows], q_pos[q_rows]
    # keys beyond the last query position are invisible to every row: leave them out
    n_keys = int(q_pos.max()) + 1
    k, v = to64(inputs["k"][:n_keys]), to64(inputs["v"][:n_keys])
    kv_pos = np.arange(n_keys, dtype=np.int64)
    r = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, w.scale, w.kv_of_q)
    o, lse = oracle.attn_fwd(q, q_pos, k, v, kv_pos, w.scale, w.kv_of_q)
    r["o"] = o
    assert np.array_equal(lse, r["lse"])
    r["n_keys"] = n_keys
    return r


def chunk_slices(w, j, x_global, n_keys):
    """Rows of a global-order [l_tot or n_keys, ...] oracle array for chunk j (zeros beyond n_keys)."""
    parts = []
    for s, n in w.chunks[j]:
        seg = np.zeros((n,) + x_global.shape[1:], dtype=x_global.dtype)
        hi = min(s + n, n_keys)
        if hi > s:
            seg[:hi - s] = x_global[s:hi]
        parts.append(seg)
    return np.concatenate(parts, axis=0)
