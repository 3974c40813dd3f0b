"""CPU oracle of the head redistribution either side of the ring: packing a device's tensor for the
ragged all-to-all and scattering what comes back.

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this module.  It shares no code with the HIP package.

What it writes out (HexiSeq Sec. 3.2, "Heterogeneous A2A with per-rank split tables" and "Sub-ring KV
exchange"; App. A.4, A2A volume equation): before the all-to-all a device holds its pre-A2A sequence
shard with all heads, ``x[s, N, d]`` (token-major, heads packed, d contiguous).  Rank j of the group is
assigned a list of heads (n_j of them, not necessarily adjacent); the part of x that goes to rank j is
``x[:, heads_j, :]``, stored contiguously as ``[s, n_j, d]``, and the send buffer is these parts one
after the other in rank order: s * n_j * d elements for rank j, the volume the cost model charges per
tensor.  The reverse direction receives one such part per rank and puts the heads back in place.
Pure data movement: results are exact, any element type.
"""
import numpy as np


def a2a_pack_loops(x, head_lists):
    """The definition, one element at a time (tiny inputs only)."""
    s, n, d = x.shape
    out = []
    for heads in head_lists:              # destination ranks in order
        for t in range(s):                # tokens of the shard
            for h in heads:               # the rank's heads in its own order
                for c in range(d):
                    out.append(x[t, h, c])
    return np.array(out, dtype=x.dtype)


def a2a_pack(x, head_lists):
    """Send buffer (1-D) for x[s, N, d]: for each rank its part x[:, heads, :] as [s, n_j, d]."""
    parts = [np.ascontiguousarray(x[:, list(heads), :]).reshape(-1) for heads in head_lists]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=x.dtype)


def a2a_unpack(buf, s, n_heads_total, d, head_lists, y=None):
    """Inverse: buf holds one [s, n_j, d] part per rank; head h of rank j's part goes to y[:, h, :].
    Heads that no list names keep the value they have in y (zeros if y is None)."""
    if y is None:
        y = np.zeros((s, n_heads_total, d), dtype=buf.dtype)
    off = 0
    for heads in head_lists:
        n_j = len(heads)
        part = buf[off:off + s * n_j * d].reshape(s, n_j, d)
        for i, h in enumerate(heads):
            y[:, h, :] = part[:, i, :]
        off += s * n_j * d
    return y


def part_offsets(s, d, head_lists):
    """Element offset of each rank's part in the send buffer, and the total length."""
    offs, off = [], 0
    for heads in head_lists:
        offs.append(off)
        off += s * len(heads) * d
    return offs, off
