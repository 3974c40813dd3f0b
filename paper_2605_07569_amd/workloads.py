"""Seeded synthetic workloads: shard geometry and N(0,1) inputs shaped like the paper's runs.

This module serves both the HIP library's tests/bench and the CPU oracle's tests.  It holds none of
the method's arithmetic: only which global token ranges and heads a device owns, which KV chunks
stream past it (HexiSeq Sec. 3.2: uneven group lengths L_k, per-rank head counts n_d; App. A.4: one
source KV block per ring step), and seeded random tensors.  The paper trains on tokenised text; the
attention cost and correctness do not depend on token identity, so N(0,1) tensors stand in for it.

A segment is ``(start, length)`` in global token positions.  A shard (or a chunk) is a list of
segments in ascending order; its rows are the segments' tokens packed back to back.
"""
from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import torch

K = 1024
Seg = Tuple[int, int]

TENSOR_IDS = {"q": 0, "k": 1, "v": 2, "d_o": 3, "cuts": 9}


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "bf16" | "f32": element type of q, k, v, dO
    n_q_heads: int                  # local (assigned) heads
    n_kv_heads: int
    head_dim: int
    l_tot: int                      # global sequence length
    q_segs: List[Seg]               # this device's query shard
    chunks: List[List[Seg]]         # KV chunk list in ring order, each a segment list
    k_scale: float = 1.0            # K is multiplied by this before rounding to dtype
    kv_of_q: Optional[List[int]] = None  # None: q head h reads kv head h // (nq / nkv)
    note: str = ""
    q_head_ids: Optional[List[int]] = None   # global id of every local q head (None: the local index); only the
    kv_head_ids: Optional[List[int]] = None  # synthetic values depend on it: a head's values follow it across shards

    @property
    def lq(self):
        return sum(n for _, n in self.q_segs)

    @property
    def scale(self):
        return 1.0 / float(self.head_dim) ** 0.5

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


def zigzag_segs(rank: int, n_ranks: int, l_tot: int) -> List[Seg]:
    """Load-balanced causal layout: 2R equal blocks, rank r owns blocks r and 2R-1-r."""
    blk = l_tot // (2 * n_ranks)
    assert blk * 2 * n_ranks == l_tot
    return [(rank * blk, blk), ((2 * n_ranks - 1 - rank) * blk, blk)]


def _seeded_cuts(seed: int, lo: int, hi: int, n_parts: int, min_len: int, quantum: int) -> List[int]:
    """n_parts-1 cut points, multiples of `quantum` strictly inside (lo, hi), every part >= min_len.

    Rejection sampling from a torch CPU generator seeded with (seed, tensor id "cuts")."""
    g = torch.Generator().manual_seed(seed * 16 + TENSOR_IDS["cuts"])
    n_slots = (hi - lo) // quantum
    for _ in range(10000):
        cuts = sorted((lo + quantum * int(c)) for c in
                      (torch.randint(1, n_slots, (n_parts - 1,), generator=g)).tolist())
        edges = [lo] + cuts + [hi]
        if all(b - a >= min_len for a, b in zip(edges[:-1], edges[1:])):
            return cuts
    raise RuntimeError("cut sampling did not converge")


def config(idx: int, seed: int = 20260507, shrink: int = 1) -> Workload:
    """The five shard configurations (idx 1..5).  `shrink` divides every token count (shape-preserving
    minis for full-tensor oracle comparison); head counts, head_dim and chunk counts are unchanged."""
    s = shrink
    if idx == 1:
        w = Workload("cfg1_tiny_fp32", "f32", 4, 4, 64, 2 * K // s, [(K // s, K // s)],
                     [[(0, K // s)], [(K // s, K // s)]], note="tokens 1024..2047 of 2048, 2 chunks")
    elif idx == 2:
        lt, r = 128 * K // s, 8
        w = Workload("cfg2_3b_zigzag", "bf16", 24, 8, 128, lt, zigzag_segs(0, r, lt),
                     [zigzag_segs(j, r, lt) for j in range(r)],
                     note="128K zigzag CP over 8 shards, rank 0 (blocks 0 and 15), chunk j = rank j's pair")
    elif idx == 3:
        lt = 256 * K // s
        fixed = [20 * K // s, 12 * K // s, 40 * K // s, 24 * K // s]
        cuts = _seeded_cuts(seed, 96 * K // s, lt, 4, 8 * K // s, K // s)
        edges = [0, fixed[0], fixed[0] + fixed[1], sum(fixed[:3]), sum(fixed)] + cuts + [lt]
        shards = [(a, b - a) for a, b in zip(edges[:-1], edges[1:])]
        w = Workload("cfg3_8b_asym", "bf16", 12, 3, 128, lt, [shards[2]], [[sh] for sh in shards],
                     note="256K cut into 8 uneven shards; owns the 40K shard at 32K and 12 of 32 q heads")
    elif idx == 4:
        lt, r = 512 * K // s, 16
        w = Workload("cfg4_8b_long", "bf16", 32, 8, 128, lt, zigzag_segs(3, r, lt),
                     [zigzag_segs(j, r, lt) for j in range(r)], k_scale=3.0,
                     note="512K zigzag CP over 16 shards, rank 3, K scaled x3")
    elif idx == 5:
        lt, c = 1024 * K // s, 32 * K // s
        w = Workload("cfg5_70b_hp", "bf16", 8, 1, 128, lt, [(480 * K // s, c)],
                     [[(j * c, c)] for j in range(32)],
                     note="1M tokens; one HP group (8 q / 1 kv head), 32K query shard at 480K, 32 chunks")
    else:
        raise ValueError("config index must be 1..5")
    if s != 1:
        w = replace(w, name=w.name + f"_div{s}")
    return w


def from_schedule(groups, l_group, n_heads, device: int, head_dim: int = 128, q_per_kv: int = 1, dtype: str = "bf16") -> Workload:
    """The attention share a schedule gives one device (Sec. 4.1: A2A groups in ring order, group sequence
    lengths L_k, per-rank head counts n_d): group k holds the sequence block [sum_{k'<k} L_k', + L_k) after the
    all-to-all, the device holds its contiguous range of n_d q heads (heads lie over a group's devices in device
    order), and the ring delivers the blocks of groups k, k-1, ... (mod K).  With GQA (q_per_kv q heads per kv
    head) the range may cut through a kv group: the kv heads it touches are held locally and kv_of_q maps onto them."""
    k = next(i for i, g in enumerate(groups) if device in g)
    starts = [sum(l_group[:i]) for i in range(len(groups))]
    lo = sum(n_heads[d] for d in groups[k] if d < device)
    q_heads = list(range(lo, lo + n_heads[device]))
    kv_global = sorted({h // q_per_kv for h in q_heads})
    kv_of_q = [kv_global.index(h // q_per_kv) for h in q_heads]
    chunks = [[(starts[(k - t) % len(groups)], l_group[(k - t) % len(groups)])] for t in range(len(groups))]
    return Workload(f"sched_dev{device}", dtype, len(q_heads), len(kv_global), head_dim, sum(l_group), [(starts[k], l_group[k])], chunks,
                    kv_of_q=kv_of_q, note=f"device {device} of a scheduled plan: group {k} of {len(groups)}, q heads {lo}..{lo + len(q_heads) - 1}",
                    q_head_ids=q_heads, kv_head_ids=kv_global)


def contiguous_chunks(w: Workload, n_chunks: int) -> Workload:
    """Alternative chunking of the same key set: n equal contiguous chunks at offsets j*Lc."""
    lc = w.l_tot // n_chunks
    assert lc * n_chunks == w.l_tot
    return replace(w, name=w.name + "_contig", chunks=[[(j * lc, lc)] for j in range(n_chunks)])


VALUE_BLOCK = 1024     # tokens per independently seeded block of a synthetic tensor
_M64 = (1 << 64) - 1


def _block_seed(seed: int, tensor_id: int, block: int, head: int) -> int:
    """A 63-bit generator seed that is a fixed function of (run seed, tensor, token block, global head)."""
    x = (seed * 0x9E3779B97F4A7C15 + (tensor_id + 1) * 0xBF58476D1CE4E5B9 + (block + 1) * 0x94D049BB133111EB + (head + 1) * 0xD6E8FEB86659FD93) & _M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _M64
    x ^= x >> 31
    return x & ((1 << 63) - 1)


def global_rows(seed: int, tensor_id: int, head_ids: List[int], head_dim: int, segs: List[Seg], dtype, scale: float = 1.0) -> torch.Tensor:
    """Rows of the synthetic global tensor [token, global head, d] for the token ranges `segs` and the heads
    `head_ids`, packed back to back: [rows, len(head_ids), d] in `dtype`.  The values are N(0,1) (times `scale`,
    then rounded to nearest even), drawn per (block of VALUE_BLOCK tokens, head) from a torch CPU generator whose seed
    is a function of (seed, tensor, block, head) alone: every shard of one sequence, whatever its token range and head
    subset, sees the same value at the same (token, head, column)."""
    total = sum(n for _, n in segs)
    out = torch.empty((total, len(head_ids), head_dim), dtype=dtype)
    pieces = []          # (first output row, block, first and last+1 token of the block taken)
    r0 = 0
    for s0, n in segs:
        pos = s0
        while pos < s0 + n:
            b = pos // VALUE_BLOCK
            lo = pos - b * VALUE_BLOCK
            hi = min(VALUE_BLOCK, s0 + n - b * VALUE_BLOCK)
            pieces.append((r0, b, lo, hi))
            r0 += hi - lo
            pos += hi - lo

    def fill(piece):
        row, b, lo, hi = piece
        g = torch.Generator()
        for i, h in enumerate(head_ids):
            g.manual_seed(_block_seed(seed, tensor_id, b, int(h)))
            blk = torch.randn((VALUE_BLOCK, head_dim), generator=g, dtype=torch.float32)[lo:hi]
            if scale != 1.0:
                blk = blk * scale
            out[row:row + (hi - lo), i] = blk.to(dtype)

    if len(pieces) >= 16:      # the pieces write disjoint rows: a few host threads share them
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, pieces))
    else:
        for piece in pieces:
            fill(piece)
    return out


def make_inputs(w: Workload, seed: int = 20260507):
    """q, d_o: [Lq, nq, d] (the shard's rows); k, v: [l_tot, nkv, d] in GLOBAL token order -- CPU tensors of w's dtype.

    Every tensor is a slice of a synthetic global tensor (see global_rows): N(0,1), K scaled by w.k_scale, rounded
    (nearest-even) to the workload dtype."""
    dt = w.torch_dtype
    q_ids = w.q_head_ids if w.q_head_ids is not None else list(range(w.n_q_heads))
    kv_ids = w.kv_head_ids if w.kv_head_ids is not None else list(range(w.n_kv_heads))
    q = global_rows(seed, TENSOR_IDS["q"], q_ids, w.head_dim, w.q_segs, dt)
    d_o = global_rows(seed, TENSOR_IDS["d_o"], q_ids, w.head_dim, w.q_segs, dt)
    k = global_rows(seed, TENSOR_IDS["k"], kv_ids, w.head_dim, [(0, w.l_tot)], dt, scale=w.k_scale)
    v = global_rows(seed, TENSOR_IDS["v"], kv_ids, w.head_dim, [(0, w.l_tot)], dt)
    return dict(q=q, k=k, v=v, d_o=d_o)


def gather_rows(x: torch.Tensor, segs: List[Seg]) -> torch.Tensor:
    """Rows of a global-order tensor for a segment list, packed back to back (a copy)."""
    if len(segs) == 1:
        s, n = segs[0]
        return x[s:s + n].contiguous()
    return torch.cat([x[s:s + n] for s, n in segs], dim=0).contiguous()


def seg_positions(segs: List[Seg]) -> torch.Tensor:
    return torch.cat([torch.arange(s, s + n, dtype=torch.int64) for s, n in segs])
