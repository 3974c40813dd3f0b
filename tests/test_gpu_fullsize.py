"""Full-size parity: configurations 2-5 at their real sizes (and configuration 2 with 64-column heads), in the
launch configuration bench.py times.

The oracle cannot recompute a whole full-size shard, so:
  (i)   o, lse and dq are row-local: at least 512 sampled (row, head subset) pairs -- the first / last rows of
        every segment, rows around tile boundaries, half of the rest among the first 1024 rows of each segment
        (the rows with the fewest visible keys and the most sharply peaked softmax), the others uniform over the
        shard -- are recomputed in fp64 against all their visible keys and compared with the full GPU run;
  (ii)  dk, dv need every shard row, so they are compared in full on a q-SUB-SHARD run: the library is called
        with a q range made of scattered short segments of the real shard (true offsets, true chunk list, one
        GQA group taken as a strided view of the real tensors), for which the full oracle is affordable;
  (iii) dk, dv of the TIMED launch itself, element by element: the last keys of the shard's last segment are
        visible to the last shard rows only, so the oracle over those rows x all heads gives the exact dk / dv of
        those keys (all kv heads) as the full-size launch must have written them;
  (iv)  the full launch of one remote chunk against other launches of the same kernel: the sum of the dk / dv of
        a partition of the shard into two sub-shards (additivity over query rows), and the same launch with a
        different head-run length (other workgroup shapes, XCD splits and atomics use), every element;
  (v)   properties that hold at any size: sum_j dV_j = sum_i dO_i per kv head (rows of P sum to 1) and
        sum <q, dq> = sum <k, dk>.
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
TRIPLE_BUDGET = 1.0e8   # (row, key, head) triples per oracle call of parts (ii) and (iii): about 15 s on 16 cores
N_SAMPLED_ROWS = 512


def _sample_rows(w, n_target):
    """Structured rows of every segment, then half of the remainder from the first 1024 rows of each segment and
    half uniformly over the shard.  Packed row indices, ascending."""
    rows, off = set(), 0
    rng = np.random.default_rng(5)
    early = []
    for s, n in w.q_segs:
        for r in (0, 1, 31, 32, 63, 64, 127, 128, 129, 255, 256, 257, n // 2, n - 257, n - 256, n - 129, n - 128, n - 2, n - 1):
            if 0 <= r < n:
                rows.add(off + r)
        early.append(off + np.arange(min(n, 1024)))
        off += n
    early = np.concatenate(early)
    need = max(0, n_target - len(rows))
    pool = np.setdiff1d(early, np.fromiter(rows, dtype=np.int64))
    rows.update(int(x) for x in rng.choice(pool, size=min(len(pool), need // 2), replace=False))
    pool = np.setdiff1d(np.arange(w.lq), np.fromiter(rows, dtype=np.int64))
    rows.update(int(x) for x in rng.choice(pool, size=min(len(pool), max(0, n_target - len(rows))), replace=False))
    return np.array(sorted(rows), dtype=np.int64)


def _kv_of(w, h):
    return w.kv_of_q[h] if w.kv_of_q else h // (w.n_q_heads // w.n_kv_heads)


def _locate(w, pos):
    """(chunk index, packed row within the chunk) of the key at global position pos."""
    for j, ch in enumerate(w.chunks):
        r0 = 0
        for s, n in ch:
            if s <= pos < s + n:
                return j, r0 + (pos - s)
            r0 += n
    raise ValueError(pos)


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

    # (v) properties at full size (fp64 sums on the GPU tensors)
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

    # (i) sampled (row, head subset) pairs of the full run, in groups of rows of similar position
    rows = _sample_rows(w, N_SAMPLED_ROWS)
    assert len(rows) >= N_SAMPLED_ROWS
    rng = np.random.default_rng(17)
    got = {n: [] for n in ("o", "lse", "delta", "dq")}
    want = {n: [] for n in got}
    n_pairs_checked = 0
    groups = [rows[i:i + 64] for i in range(0, len(rows), 64)]
    print(f"  oracle on {len(rows)} sampled rows in {len(groups)} groups, 1-2 heads each", flush=True)
    for g_rows in groups:
        q_pos = q_pos_all[g_rows]
        n_keys = int(q_pos.max()) + 1
        n_h = 2 if n_keys <= 200 * 1024 else 1       # rows that see several hundred thousand keys: one head each
        heads = sorted(int(h) for h in rng.choice(nq, size=min(n_h, nq), replace=False))
        kvs = sorted({_kv_of(w, h) for h in heads})
        kv_map = [kvs.index(_kv_of(w, h)) for h in heads]
        k64, v64 = to64(inputs["k"][:n_keys][:, kvs]), to64(inputs["v"][:n_keys][:, kvs])
        q64, g64 = to64(inputs["q"][g_rows][:, heads]), to64(inputs["d_o"][g_rows][:, heads])
        kv_pos = np.arange(n_keys, dtype=np.int64)
        ref = oracle.attn_bwd(q64, q_pos, k64, v64, kv_pos, g64, w.scale, kv_map)
        o_ref, _ = oracle.attn_fwd(q64, q_pos, k64, v64, kv_pos, w.scale, kv_map)
        rt, ht = torch.as_tensor(g_rows, device=DEV), torch.as_tensor(heads, device=DEV)
        got["o"].append(run.o[rt][:, ht].cpu().numpy()); want["o"].append(o_ref)
        got["dq"].append(run.dq[rt][:, ht].cpu().numpy()); want["dq"].append(ref["dq"])
        got["lse"].append(run.lse[ht][:, rt].cpu().numpy().T); want["lse"].append(ref["lse"].T)
        got["delta"].append(run.delta[ht][:, rt].cpu().numpy().T); want["delta"].append(ref["delta"].T)
        n_pairs_checked += len(g_rows) * len(heads)
        del ref, o_ref, k64, v64
    print(f"    {n_pairs_checked} (row, head) pairs", flush=True)
    cat = lambda xs: np.concatenate([np.asarray(x).reshape(-1) for x in xs])
    check("o[rows]", cat(got["o"]), cat(want["o"]), "bf16")
    check("lse[rows]", cat(got["lse"]), cat(want["lse"]), "bf16")
    check("dq[rows]", cat(got["dq"]), cat(want["dq"]), "bf16")
    # Delta is an intermediate, not one of the five outputs: a sum of d products of dO with o, so its absolute error
    # is up to sqrt(d) |dO| times that of o; its effect is covered by the flat bounds on dq above and dk below
    check("delta[rows] (intermediate)", cat(got["delta"]), cat(want["delta"]), "bf16", abs_factor=float(d) ** 0.5)

    # (ii) q-sub-shard run: scattered 16-row segments of the real shard, one GQA group (strided views)
    avg_keys = float(np.mean(q_pos_all + 1))
    n_rows = int(min(192, max(32, TRIPLE_BUDGET / (avg_keys * grp))))
    n_seg = max(2, min(12, n_rows // 16))
    rng = np.random.default_rng(9)
    lq = w.lq
    starts = sorted(int(x) for x in rng.choice(lq // 16 - 1, size=n_seg - 2, replace=False) * 16 + 3) if n_seg > 2 else []
    starts = sorted(set([0] + starts + [lq - 16]))
    sub_rows = np.concatenate([np.arange(s, s + 16) for s in starts])

    def segments_of(packed_rows):
        """packed shard rows (ascending) -> global segments (a run may straddle two shard segments; split it then)"""
        pos = q_pos_all[packed_rows]
        segs, s0 = [], 0
        for i in range(1, len(pos) + 1):
            if i == len(pos) or pos[i] != pos[i - 1] + 1:
                segs.append((int(pos[s0]), i - s0))
                s0 = i
        assert len(segs) <= hexi.HEXI_MAX_SEGS
        return segs

    sub_pos = q_pos_all[sub_rows]
    segs = segments_of(sub_rows)
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
    del ref, dk_all, dv_all, dk_ref, dv_ref, dks, dvs

    # (iii) dk / dv of the timed launch: the last n keys of the shard's last segment see only the last n shard rows
    p_end = int(q_pos_all.max()) + 1
    n_last = int(max(8, min(128, TRIPLE_BUDGET * 0.75 / (float(p_end) * nq))))
    last_rows = np.arange(lq - n_last, lq)
    assert q_pos_all[last_rows[0]] == p_end - n_last          # the shard's last segment is at least n_last long
    print(f"  oracle on the last {n_last} shard rows x all {nq} heads x {p_end} keys (dk / dv of the last {n_last} keys)", flush=True)
    ref = oracle.attn_bwd(to64(inputs["q"][last_rows]), q_pos_all[last_rows], to64(inputs["k"][:p_end]), to64(inputs["v"][:p_end]),
                          np.arange(p_end, dtype=np.int64), to64(inputs["d_o"][last_rows]), w.scale, w.kv_of_q)
    j_diag, r_first = _locate(w, p_end - n_last)
    assert _locate(w, p_end - 1) == (j_diag, r_first + n_last - 1)
    check("dk[last keys] (timed launch)", run.dk[j_diag][r_first:r_first + n_last].cpu(), ref["dk"][p_end - n_last:], "bf16")
    check("dv[last keys] (timed launch)", run.dv[j_diag][r_first:r_first + n_last].cpu(), ref["dv"][p_end - n_last:], "bf16")
    del ref

    # (iv) one remote chunk: full launch = sum of the launches of two sub-shards (the scattered rows of (ii), all
    # heads, and the rest of the shard), and = the same launch with another head-run length.  fp32 summation order
    # is all that differs, so the bounds are far below the output tolerance.
    def remote(ch):
        return not any(ks < qs + qn and qs < ks + kn for qs, qn in w.q_segs for ks, kn in ch) and ch[0][0] <= q_pos_all.max()
    j_r = next(j for j, ch in enumerate(w.chunks) if remote(ch))
    kc, vc = run.k[j_r], run.v[j_r]
    dk_full, dv_full = run.dk[j_r], run.dv[j_r]
    acc_k, acc_v = torch.zeros_like(dk_full), torch.zeros_like(dv_full)
    rest = np.setdiff1d(np.arange(lq), sub_rows)
    for part in (sub_rows, rest):
        pt = torch.as_tensor(part, device=DEV)
        q_p, do_p = run.q[pt].contiguous(), run.d_o[pt].contiguous()
        lse_p, delta_p = run.lse[:, pt].contiguous(), run.delta[:, pt].contiguous()
        hexi.hexi_attn_bwd_chunk(hexi.desc_for(q_p, kc, w.scale, w.kv_of_q), segments_of(part), w.chunks[j_r], q_p, kc, vc, None, do_p,
                                 lse_p, delta_p, None, acc_k, acc_v, flags=hexi.HEXI_ACCUMULATE | hexi.HEXI_SKIP_DQ)
    torch.cuda.synchronize()

    def close(name, a, b):
        err = float((a.double() - b.double()).abs().max())
        rel = float((a.double() - b.double()).norm() / b.double().norm())
        print(f"    {name}: max_abs={err:.3e} rel_l2={rel:.3e}", flush=True)
        assert err <= 2e-3 and rel <= 1e-4, name

    print(f"  chunk {j_r}: full launch vs the sum over two sub-shards ({len(sub_rows)} + {len(rest)} rows)", flush=True)
    close("dk additivity", acc_k, dk_full)
    close("dv additivity", acc_v, dv_full)
    del acc_k, acc_v
    try:
        for run_len in (1, grp):
            dk2, dv2 = torch.empty_like(dk_full), torch.empty_like(dv_full)
            hexi.hexi_set_dkdv_run_len(run_len)
            hexi.hexi_attn_bwd_chunk(run.desc[j_r], w.q_segs, w.chunks[j_r], run.q, kc, vc, None, run.d_o, run.lse, run.delta,
                                     None, dk2, dv2, flags=hexi.HEXI_SKIP_DQ)
            torch.cuda.synchronize()
            close(f"dk, head runs of {run_len}", dk2, dk_full)
            close(f"dv, head runs of {run_len}", dv2, dv_full)
            del dk2, dv2
    finally:
        hexi.hexi_set_dkdv_run_len(0)


@pytest.mark.parametrize("idx", [2, 4])
def test_full_size_contiguous_chunk_replay(idx):
    """The other reading of "KV chunk" for the zigzag configurations: the same keys as equal contiguous chunks.  At full
    size: sampled rows of o, lse, dq against the oracle, and every element of o, lse, dq and (per global key) dk, dv
    against the zigzag-pair replay of the same shard, which the test above ties to the oracle."""
    w = wl.config(idx)
    wc = wl.contiguous_chunks(w, len(w.chunks))
    print(f"\n[{wc.name}] generating inputs", flush=True)
    inputs = wl.make_inputs(w)
    q_pos_all = wl.seg_positions(w.q_segs).numpy()
    nq, nkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim

    def global_order(run, ww):
        """dk, dv of all chunks scattered back to global key order (float32 [l_tot, nkv, d] on the GPU)."""
        gk = torch.zeros((ww.l_tot, nkv, d), dtype=torch.float32, device=DEV)
        gv = torch.zeros_like(gk)
        for j, ch in enumerate(ww.chunks):
            r0 = 0
            for s, n in ch:
                gk[s:s + n] = run.dk[j][r0:r0 + n]
                gv[s:s + n] = run.dv[j][r0:r0 + n]
                r0 += n
        return gk, gv

    run = replay.ShardRun(w, inputs, DEV)
    run.step()
    torch.cuda.synchronize()
    o_z, lse_z, dq_z = run.o.clone(), run.lse.clone(), run.dq.clone()
    dk_z, dv_z = global_order(run, w)
    del run
    torch.cuda.empty_cache()
    run = replay.ShardRun(wc, inputs, DEV)
    run.step()
    torch.cuda.synchronize()
    print("  both replays done", flush=True)
    dk_c, dv_c = global_order(run, wc)
    for name, a, b in (("o", run.o, o_z), ("lse", run.lse, lse_z), ("dq", run.dq, dq_z), ("dk", dk_c, dk_z), ("dv", dv_c, dv_z)):
        fin = torch.isfinite(b)
        assert torch.equal(torch.isfinite(a), fin)
        err = float((a[fin].double() - b[fin].double()).abs().max())
        rel = float((a[fin].double() - b[fin].double()).norm() / b[fin].double().norm())
        print(f"    {name}: contiguous vs zigzag-pair chunks: max_abs={err:.3e} rel_l2={rel:.3e}", flush=True)
        assert err <= 2e-2 and rel <= 5e-3, name
    del o_z, lse_z, dq_z, dk_z, dv_z, dk_c, dv_c
    # sampled rows against the oracle (one head each; half of them among the first 1024 rows of each segment)
    rows = _sample_rows(w, 128)
    rng = np.random.default_rng(23)
    got = {n: [] for n in ("o", "lse", "dq")}
    want = {n: [] for n in got}
    for g_rows in [rows[i:i + 64] for i in range(0, len(rows), 64)]:
        q_pos = q_pos_all[g_rows]
        n_keys = int(q_pos.max()) + 1
        h = int(rng.integers(0, nq))
        kh = _kv_of(w, h)
        k64, v64 = to64(inputs["k"][:n_keys][:, [kh]]), to64(inputs["v"][:n_keys][:, [kh]])
        q64, g64 = to64(inputs["q"][g_rows][:, [h]]), to64(inputs["d_o"][g_rows][:, [h]])
        kv_pos = np.arange(n_keys, dtype=np.int64)
        ref = oracle.attn_bwd(q64, q_pos, k64, v64, kv_pos, g64, w.scale, [0])
        o_ref, _ = oracle.attn_fwd(q64, q_pos, k64, v64, kv_pos, w.scale, [0])
        rt = torch.as_tensor(g_rows, device=DEV)
        got["o"].append(run.o[rt][:, h].cpu().numpy()); want["o"].append(o_ref[:, 0])
        got["dq"].append(run.dq[rt][:, h].cpu().numpy()); want["dq"].append(ref["dq"][:, 0])
        got["lse"].append(run.lse[h][rt].cpu().numpy()); want["lse"].append(ref["lse"][0])
    cat = lambda xs: np.concatenate([np.asarray(x).reshape(-1) for x in xs])
    print(f"  oracle on {len(rows)} sampled rows, one head each", flush=True)
    for n in ("o", "lse", "dq"):
        check(f"{n}[rows] (contiguous chunks)", cat(got[n]), cat(want[n]), "bf16")
