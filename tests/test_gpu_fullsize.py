"""Full-size parity: configurations 2-5 at their real sizes (and configuration 2 with 64-column heads), in the
launch configuration bench.py times.

The oracle cannot recompute a whole full-size shard, so:
  (i)  o, lse and dq are row-local: sampled rows (first / last rows of every segment, rows around tile
       boundaries, evenly spaced rows) x all local heads are recomputed one by one in fp64 against all
       their visible keys and compared with the rows of the full GPU run;
  (ii) dk, dv need every shard row, so they are compared in full on a q-SUB-SHARD run: the library is
       called with a q range made of scattered short segments of the real shard (true offsets, true
       chunk list, one GQA group taken as a strided view of the real tensors), for which the full
       oracle is affordable; every dk/dv element of every chunk is compared;
  (iii) properties that hold at any size tie the full-size dk, dv to the inputs:
       sum_j dV_j = sum_i dO_i per kv head (rows of P sum to 1) and sum <q, dq> = sum <k, dk>.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07569_amd import hexi, replay
from paper_2605_07569_amd import workloads as wl
from parity_util import check, chunk_slices, to64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TRIPLE_BUDGET = 1.0e8   # (row, key, head) triples per oracle call: seconds to tens of seconds on 16 cores


def _sample_rows(w, n_target):
    rows, off = set(), 0
    for s, n in w.q_segs:
        for r in (0, 1, 63, 64, 127, 128, 129, n // 2, n - 129, n - 128, n - 2, n - 1):
            if 0 <= r < n:
                rows.add(off + r)
        off += n
    rng = np.random.default_rng(5)
    lq = w.lq
    extra = max(0, n_target - len(rows))
    rows.update(int(x) for x in rng.choice(lq, size=extra, replace=False))
    return np.array(sorted(rows), dtype=np.int64)


@pytest.mark.parametrize("idx,head_dim", [(2, 128), (3, 128), (4, 128), (5, 128), (2, 64)])
def test_full_size_sampled_rows_subshard_and_properties(idx, head_dim):
    w = wl.config(idx)
    if head_dim != w.head_dim:      # variant: the same shard with 64-column heads (the launch `bench.py --head-dim 64` times)
        import dataclasses
        w = dataclasses.replace(w, head_dim=head_dim, name=f"{w.name}_d{head_dim}")
    print(f"\n[{w.name}] generating inputs", flush=True)
    inputs = wl.make_inputs(w)
    q_pos_all = wl.seg_positions(w.q_segs).numpy()
    nq, nkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    grp = nq // nkv
    run = replay.ShardRun(w, inputs, DEV)
    run.step()
    torch.cuda.synchronize()
    print("  GPU replay done", flush=True)

    # (iii) properties at full size (fp64 sums on the GPU tensors)
    dv_sum = sum(x.double().sum(0) for x in run.dv)                      # [nkv, d]
    do_sum = run.d_o.double().sum(0).reshape(nkv, grp, d).sum(1)         # default head map: groups are contiguous
    rel = float((dv_sum - do_sum).norm() / do_sum.norm())
    print(f"    sum_j dV_j vs sum_i dO_i: rel {rel:.3e}", flush=True)
    assert rel < 5e-3
    lhs = float((run.q.double() * run.dq.double()).sum())
    rhs = float(sum((kc.double() * dk.double()).sum() for kc, dk in zip(run.k, run.dk)))
    scale_ref = float(sum((kc.double() * dk.double()).abs().sum() for kc, dk in zip(run.k, run.dk)))
    print(f"    <q,dq> = {lhs:.6e}  <k,dk> = {rhs:.6e}  (sum |k dk| = {scale_ref:.3e})", flush=True)
    assert abs(lhs - rhs) <= 5e-3 * scale_ref
    n_future = sum(1 for ch in w.chunks if ch[0][0] > q_pos_all.max())
    for j, ch in enumerate(w.chunks):
        if ch[0][0] > q_pos_all.max():
            assert not run.dk[j].any() and not run.dv[j].any()
    print(f"    {n_future} chunks wholly in the future: zero dk/dv", flush=True)

    # (i) sampled rows of the full run
    avg_keys = float(np.mean(q_pos_all + 1))
    rows = _sample_rows(w, max(24, int(TRIPLE_BUDGET / (avg_keys * nq))))
    q_pos = q_pos_all[rows]
    n_keys = int(q_pos.max()) + 1
    k64, v64 = to64(inputs["k"][:n_keys]), to64(inputs["v"][:n_keys])
    kv_pos = np.arange(n_keys, dtype=np.int64)
    print(f"  oracle on {len(rows)} sampled rows x {nq} heads x up to {n_keys} keys", flush=True)
    ref = oracle.attn_bwd(to64(inputs["q"][rows]), q_pos, k64, v64, kv_pos, to64(inputs["d_o"][rows]), w.scale)
    o_ref, lse_ref = oracle.attn_fwd(to64(inputs["q"][rows]), q_pos, k64, v64, kv_pos, w.scale)
    rt = torch.as_tensor(rows, device=DEV)
    check("o[rows]", run.o[rt].cpu(), o_ref, "bf16")
    check("lse[rows]", run.lse[:, rt].cpu(), lse_ref, "bf16")
    check("delta[rows]", run.delta[:, rt].cpu(), ref["delta"], "bf16", abs_factor=float(d) ** 0.5)
    check("dq[rows]", run.dq[rt].cpu(), ref["dq"], "bf16")
    del ref, o_ref

    # (ii) q-sub-shard run: scattered 16-row segments of the real shard, one GQA group (strided views)
    n_rows = int(min(192, max(32, TRIPLE_BUDGET / (avg_keys * grp))))
    n_seg = max(2, min(12, n_rows // 16))
    rng = np.random.default_rng(9)
    lq = w.lq
    starts = sorted(int(x) for x in rng.choice(lq // 16 - 1, size=n_seg - 2, replace=False) * 16 + 3) if n_seg > 2 else []
    starts = sorted(set([0] + starts + [lq - 16]))
    sub_rows = np.concatenate([np.arange(s, s + 16) for s in starts])
    # packed rows -> global segments (a 16-row run may straddle two shard segments; split it then)
    sub_pos = q_pos_all[sub_rows]
    segs, s0 = [], 0
    for i in range(1, len(sub_pos) + 1):
        if i == len(sub_pos) or sub_pos[i] != sub_pos[i - 1] + 1:
            segs.append((int(sub_pos[s0]), i - s0))
            s0 = i
    assert len(segs) <= hexi.HEXI_MAX_SEGS
    st = torch.as_tensor(sub_rows, device=DEV)
    q_sub = run.q[st][:, :grp]            # strided view: first group's q heads
    do_sub = run.d_o[st][:, :grp]
    f32 = dict(dtype=torch.float32, device=DEV)
    o_s = torch.zeros((len(sub_rows), grp, d), **f32)
    lse_s = torch.full((grp, len(sub_rows)), float("-inf"), **f32)
    delta_s = torch.empty_like(lse_s)
    dq_s = torch.zeros_like(o_s)
    dks, dvs = [], []
    descs = []
    for j, ch in enumerate(w.chunks):
        kc, vc = run.k[j][:, :1], run.v[j][:, :1]
        desc = hexi.desc_for(q_sub, kc, w.scale)
        descs.append(desc)
        hexi.hexi_attn_fwd_chunk(desc, segs, ch, q_sub, kc, vc, o_s, lse_s, flags=hexi.HEXI_ACCUMULATE)
    for j, ch in enumerate(w.chunks):
        kc, vc = run.k[j][:, :1], run.v[j][:, :1]
        dk = torch.empty((kc.shape[0], 1, d), **f32)
        dv = torch.empty_like(dk)
        hexi.hexi_attn_bwd_chunk(descs[j], segs, ch, q_sub, kc, vc, o_s, do_sub, lse_s, delta_s, dq_s, dk, dv,
                                 flags=hexi.HEXI_COMPUTE_DELTA if j == 0 else 0)
        dks.append(dk); dvs.append(dv)
    torch.cuda.synchronize()
    n_keys = int(sub_pos.max()) + 1
    print(f"  oracle on a {len(sub_rows)}-row / {len(segs)}-segment sub-shard x {grp} heads x {n_keys} keys", flush=True)
    ref = oracle.attn_bwd(to64(inputs["q"][sub_rows][:, :grp]), sub_pos, to64(inputs["k"][:n_keys, :1]),
                          to64(inputs["v"][:n_keys, :1]), np.arange(n_keys, dtype=np.int64),
                          to64(inputs["d_o"][sub_rows][:, :grp]), w.scale)
    check("sub.lse", lse_s.cpu(), ref["lse"], "bf16")
    check("sub.dq", dq_s.cpu(), ref["dq"], "bf16")
    dk_all = np.concatenate([x.cpu().numpy() for x in dks])
    dv_all = np.concatenate([x.cpu().numpy() for x in dvs])
    dk_ref = np.concatenate([chunk_slices(w, j, ref["dk"], n_keys) for j in range(len(w.chunks))])
    dv_ref = np.concatenate([chunk_slices(w, j, ref["dv"], n_keys) for j in range(len(w.chunks))])
    check("sub.dk (all keys)", dk_all, dk_ref, "bf16")
    check("sub.dv (all keys)", dv_all, dv_ref, "bf16")
