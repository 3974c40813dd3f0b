"""GPU parity: the HIP library, called through the C ABI, against the fp64 CPU oracle.

Tier 0: configuration 1 (fp32) in full.  Tier 1: shape-preserving minis of configurations 2-5
(all token counts divided, heads / head_dim / chunk structure kept), every output element.  Edge
cases: ragged lengths, many segments, strided inputs, explicit head maps, chunks in the future,
rows that see nothing, the unfused fwd + merge path, accumulate flags.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07569_amd import hexi, replay
from paper_2605_07569_amd import workloads as wl
from parity_util import check, chunk_slices, oracle_full, to64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture
def force_run_len():
    """Sets the dK/dV launcher's forced head-run length for the test and restores the automatic choice after it."""
    yield hexi.hexi_set_dkdv_run_len
    hexi.hexi_set_dkdv_run_len(0)


def _run_and_compare(w, seed=20260507, fused=True):
    """Runs the whole replay on the GPU and compares every element of every output with the oracle at the flat
    tolerances.  (Delta, an intermediate and not one of the five outputs, is a sum of d products of dO with o: its
    max-abs bound is that of o times sqrt(d); its effect on the outputs is covered by the flat bounds on dq / dk.)"""
    print(f"\n[{w.name}] lq={w.lq} heads={w.n_q_heads}/{w.n_kv_heads} d={w.head_dim} chunks={len(w.chunks)} fused={fused}", flush=True)
    inputs = wl.make_inputs(w, seed)
    run = replay.ShardRun(w, inputs, DEV, fused_merge=fused)
    run.step()
    torch.cuda.synchronize()
    ref = oracle_full(w, inputs)
    dk = np.concatenate([run.dk[j].cpu().numpy() for j in range(len(w.chunks))])
    dv = np.concatenate([run.dv[j].cpu().numpy() for j in range(len(w.chunks))])
    dk_ref = np.concatenate([chunk_slices(w, j, ref["dk"], ref["n_keys"]) for j in range(len(w.chunks))])
    dv_ref = np.concatenate([chunk_slices(w, j, ref["dv"], ref["n_keys"]) for j in range(len(w.chunks))])
    failures = []
    for name, got, want, fac in (("o", run.o.cpu(), ref["o"], 1.0), ("lse", run.lse.cpu(), ref["lse"], 1.0),
                                 ("delta", run.delta.cpu(), ref["delta"], float(w.head_dim) ** 0.5),
                                 ("dq", run.dq.cpu(), ref["dq"], 1.0), ("dk", dk, dk_ref, 1.0),
                                 ("dv", dv, dv_ref, 1.0)):
        try:
            check(name, got, want, w.dtype, abs_factor=fac)
        except AssertionError as e:
            failures.append(str(e))
    assert not failures, failures
    return run, inputs, ref


def test_tier0_cfg1_fp32_full():
    run, inputs, ref = _run_and_compare(wl.config(1))
    # bookkeeping: counted pairs of the replay equal the closed form
    n = sum(hexi.hexi_shard_mask(run.w.q_segs, ch, want_pos=False)["n_pairs"] for ch in run.w.chunks)
    assert n == 1573376


def test_cfg1_unfused_partials_and_merge():
    w = wl.config(1)
    inputs = wl.make_inputs(w)
    run = replay.ShardRun(w, inputs, DEV, fused_merge=False, keep_partials=True)
    run.forward()
    torch.cuda.synchronize()
    q_pos = wl.seg_positions(w.q_segs).numpy()
    q = to64(inputs["q"])
    o_acc = np.zeros_like(q)
    lse_acc = np.full((w.n_q_heads, w.lq), -np.inf)
    for j, ch in enumerate(w.chunks):
        kc, vc = to64(wl.gather_rows(inputs["k"], ch)), to64(wl.gather_rows(inputs["v"], ch))
        o_p, lse_p = oracle.attn_fwd(q, q_pos, kc, vc, wl.seg_positions(ch).numpy(), w.scale)
        check(f"o_part[{j}]", run.partials[j][0].cpu(), o_p, "f32")
        check(f"lse_part[{j}]", run.partials[j][1].cpu(), lse_p, "f32")
        o_acc, lse_acc = oracle.merge(o_acc, lse_acc, o_p, lse_p)
    check("o_merged", run.o.cpu(), o_acc, "f32")
    check("lse_merged", run.lse.cpu(), lse_acc, "f32")


@pytest.mark.parametrize("idx,shrink", [(2, 16), (3, 16), (4, 32), (5, 32)])
def test_tier1_minis_full_tensor(idx, shrink):
    # (configuration 4 scales K by 3: sharply peaked rows, whose few large dS values the dQ kernel carries with
    # their rounding residuals; every configuration is held to the same flat bounds)
    _run_and_compare(wl.config(idx, shrink=shrink))


def test_cfg2_mini_unfused_and_contiguous_chunking_agree():
    w = wl.config(2, shrink=32)
    _run_and_compare(w, fused=False)
    _run_and_compare(wl.contiguous_chunks(w, 8))


def _custom(name, dtype, nq, nkv, d, l_tot, q_segs, chunks, kv_of_q=None, k_scale=1.0):
    return wl.Workload(name, dtype, nq, nkv, d, l_tot, q_segs, chunks, k_scale=k_scale, kv_of_q=kv_of_q)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
def test_ragged_lengths_and_many_segments(dtype, d):
    # unaligned shard / chunk lengths (1000, 777, 1, 130), a shard of 4 segments, chunks of 1-3
    # segments, one chunk wholly in the future, rows that see nothing of some chunk
    q_segs = [(37, 1), (100, 130), (400, 777), (1500, 92)]
    chunks = [[(0, 777)], [(777, 1), (778, 222)], [(1000, 130), (1130, 370), (1500, 92)], [(1592, 408)]]
    w = _custom(f"ragged_{dtype}_{d}", dtype, 4, 2, d, 2000, q_segs, chunks)
    _run_and_compare(w, seed=7)


def test_explicit_head_map_and_single_rows():
    # a kv head shared by non-adjacent q heads (an HP cut through GQA groups), 1-row shard and 1-key chunk
    w = _custom("headmap", "bf16", 6, 3, 128, 600, [(0, 1), (299, 301)], [[(0, 1)], [(1, 299)], [(300, 300)]],
                kv_of_q=[2, 0, 1, 0, 2, 2])
    _run_and_compare(w, seed=11)
    w = _custom("headmap_f32", "f32", 3, 2, 64, 200, [(150, 50)], [[(0, 200)]], kv_of_q=[1, 0, 1])
    _run_and_compare(w, seed=12)


@pytest.mark.parametrize("run_len", [1, 2, 3, 8])
def test_dkdv_head_runs(run_len, force_run_len):
    # The dK/dV kernel walks runs of q heads that share a kv head in one workgroup; the launcher picks the
    # run length from the launch size, so small shapes would only ever see runs of one head.  Force the
    # length: whole groups (no atomics), runs with a remainder (3 of 5), non-adjacent heads of a group,
    # groups of unequal size, masked + full + ragged tiles in every head of a run.
    force_run_len(run_len)
    w = _custom(f"runs{run_len}", "bf16", 8, 3, 128, 700, [(150, 70), (400, 300)], [[(0, 333)], [(333, 367)]],
                kv_of_q=[0, 1, 0, 0, 2, 0, 1, 0])
    _run_and_compare(w, seed=21)
    # one group of 8 heads over several key tiles, unfused path
    w = _custom(f"runs{run_len}_hp", "bf16", 8, 1, 128, 1024, [(512, 512)], [[(0, 512)], [(512, 512)]])
    _run_and_compare(w, seed=22, fused=False)


def _random_case(rng, i, l_range=(200, 1400), max_heads=8, d_bf16=128):
    """A seeded random shard: the sequence [0, L) cut into pieces, each piece dealt to one of 1-4 chunks, the q
    shard takes 1-3 pieces; random head counts and kv map."""
    dtype = "bf16" if i % 3 else "f32"
    d = d_bf16 if dtype == "bf16" else int(rng.choice([64, 128]))
    L = int(rng.integers(*l_range))
    n_pieces = int(rng.integers(2, 9))
    cuts = sorted(set(int(c) for c in rng.integers(1, L, size=n_pieces - 1)))
    edges = [0] + cuts + [L]
    pieces = [(a, b - a) for a, b in zip(edges[:-1], edges[1:])]
    # every piece goes to exactly one chunk (the chunks together hold every key the shard can see); a chunk's
    # pieces need not be adjacent, so its segment list has holes, as a zigzag pair does
    n_chunks = int(rng.integers(1, min(4, len(pieces)) + 1))
    owner = rng.integers(0, n_chunks, size=len(pieces))
    chunks = [[p for p, o in zip(pieces, owner) if o == c] for c in range(n_chunks)]
    chunks = [c for c in chunks if c]
    rng.shuffle(chunks)                       # the ring may deliver them in any order
    own = sorted(rng.choice(len(pieces), size=min(len(pieces), int(rng.integers(1, 4))), replace=False).tolist())
    q_segs = [pieces[k] for k in own]
    nkv = int(rng.integers(1, 4))
    nq = int(rng.integers(nkv, max(nkv, max_heads) + 1))
    kv_of_q = sorted(int(x) for x in rng.integers(0, nkv, size=nq)) if rng.random() < 0.5 else [int(x) for x in rng.integers(0, nkv, size=nq)]
    return _custom(f"rand{i}_{dtype}", dtype, nq, nkv, d, L, q_segs, chunks, kv_of_q=kv_of_q)


def test_randomized_small_shards():
    rng = np.random.default_rng(20260507)
    for i in range(16):
        w = _random_case(rng, i)
        _run_and_compare(w, seed=100 + i, fused=bool(i % 2))


def test_randomized_longer_shards():
    # the same generator at lengths that span many q tiles (256 rows) and key tiles (64 / 128 keys) per workgroup
    rng = np.random.default_rng(7569)
    for i in range(8):
        w = _random_case(rng, 3 * i + 1, l_range=(2500, 6000), max_heads=4)     # bf16 cases
        _run_and_compare(w, seed=200 + i, fused=bool(i % 2))


def test_bf16_head_dim_64_minis_and_head_runs(force_run_len):
    # the bf16 kernels at head_dim 64 (the smaller models' heads): configurations 2 and 5 shrunk, heads halved to
    # 64 columns (zigzag pairs, one GQA group of 8, FULL + diagonal + EMPTY chunks), fused and unfused
    import dataclasses
    for idx, shrink in ((2, 32), (5, 64)):
        w = dataclasses.replace(wl.config(idx, shrink=shrink), head_dim=64, name=f"cfg{idx}_mini_d64")
        _run_and_compare(w, fused=(idx == 2))
    # forced dK/dV head runs: whole groups, runs with a remainder, non-adjacent heads of a group
    for run_len in (1, 3, 8):
        force_run_len(run_len)
        w = _custom(f"runs{run_len}_d64", "bf16", 8, 3, 64, 700, [(150, 70), (400, 300)], [[(0, 333)], [(333, 367)]],
                    kv_of_q=[0, 1, 0, 0, 2, 0, 1, 0])
        _run_and_compare(w, seed=31)


def test_bf16_head_dim_64_randomized_shards():
    rng = np.random.default_rng(64)
    for i in range(12):
        long_case = i >= 8     # the last four span many tiles per workgroup
        w = _random_case(rng, 3 * i + 1, l_range=(2500, 6000) if long_case else (200, 1400),
                         max_heads=4 if long_case else 8, d_bf16=64)
        _run_and_compare(w, seed=300 + i, fused=bool(i % 2))


@pytest.mark.parametrize("lq,lc", [(1, 1), (63, 65), (256, 129), (257, 300), (513, 1)])
def test_bf16_head_dim_64_workgroup_boundary_sizes(lq, lc):
    w = _custom(f"edge64_{lq}_{lc}", "bf16", 2, 1, 64, lc + lq, [(lc, lq)], [[(0, lc)], [(lc, lq)]])
    _run_and_compare(w, seed=lq * 1000 + lc + 64)


@pytest.mark.parametrize("run_len", [0, 1, 2])
def test_strided_inputs_and_accumulate_flags(run_len, force_run_len):
    # (also with forced dK/dV head runs: whole groups in one workgroup add to the running dk/dv without
    # atomics, split groups with them)
    force_run_len(run_len)
    # q/dO and k/v are slices of wider buffers (token and head strides larger than dense)
    w = _custom("strided", "bf16", 4, 2, 128, 512, [(128, 384)], [[(0, 256)], [(256, 256)]])
    inputs = wl.make_inputs(w, 5)
    dev = torch.device(DEV)
    lq, nq, nkv, d = w.lq, 4, 2, 128
    qbig = torch.zeros((lq, nq + 2, d + 64), dtype=torch.bfloat16, device=dev)
    gbig = torch.zeros_like(qbig)
    q, d_o = qbig[:, 1:1 + nq, 8:8 + d], gbig[:, 1:1 + nq, 8:8 + d]
    q.copy_(inputs["q"]); d_o.copy_(inputs["d_o"])
    o = torch.zeros((lq, nq, d), dtype=torch.float32, device=dev)
    lse = torch.full((nq, lq), float("-inf"), dtype=torch.float32, device=dev)
    delta = torch.empty_like(lse)
    dq = torch.zeros_like(o)
    ks, vs, descs = [], [], []
    for ch in w.chunks:
        kbig = torch.zeros((256, nkv + 1, d + 8), dtype=torch.bfloat16, device=dev)
        vbig = torch.zeros_like(kbig)
        kc, vc = kbig[:, :nkv, 8:], vbig[:, :nkv, 8:]
        kc.copy_(wl.gather_rows(inputs["k"], ch)); vc.copy_(wl.gather_rows(inputs["v"], ch))
        ks.append(kc); vs.append(vc)
        desc = hexi.desc_for(q, kc, w.scale)
        descs.append(desc)
        hexi.hexi_attn_fwd_chunk(desc, w.q_segs, ch, q, kc, vc, o, lse, flags=hexi.HEXI_ACCUMULATE)
    # dk/dv with HEXI_ACCUMULATE on pre-filled buffers: result = prefill + gradient
    dks = [torch.full((256, nkv, d), 0.5, dtype=torch.float32, device=dev) for _ in w.chunks]
    dvs = [torch.full((256, nkv, d), -0.25, dtype=torch.float32, device=dev) for _ in w.chunks]
    for j, ch in enumerate(w.chunks):
        flags = hexi.HEXI_ACCUMULATE | (hexi.HEXI_COMPUTE_DELTA if j == 0 else 0)
        hexi.hexi_attn_bwd_chunk(descs[j], w.q_segs, ch, q, ks[j], vs[j], o, d_o, lse, delta, dq, dks[j], dvs[j], flags=flags)
    torch.cuda.synchronize()
    ref = oracle_full(w, inputs)
    check("o", o.cpu(), ref["o"], "bf16")
    check("lse", lse.cpu(), ref["lse"], "bf16")
    check("dq", dq.cpu(), ref["dq"], "bf16")
    check("dk", torch.cat(dks).cpu().numpy() - 0.5, ref["dk"], "bf16")
    check("dv", torch.cat(dvs).cpu().numpy() + 0.25, ref["dv"], "bf16")


@pytest.mark.parametrize("d", [128, 64])
def test_dq_residuals_of_large_ds(d):
    # The dQ kernel adds the rounding residuals of a 32-key block's dS when some |dS| >= 2.  With dO scaled by 64 (exact
    # in bf16; every gradient is linear in dO) nearly every block takes that path -- masked and unmasked tiles, ragged
    # tails, both groups of a workgroup -- and dq / 64 must still match the oracle, more closely than without the scaling
    # (dS carried to fp32 accuracy instead of bf16); dk and dv, which have no such path, must come out as exactly 64 x
    # their unscaled values.
    w = _custom(f"residual_{d}", "bf16", 4, 2, d, 1500, [(60, 200), (700, 777)], [[(0, 333)], [(333, 617), (950, 27)], [(977, 523)]],
                k_scale=2.0)
    inputs = wl.make_inputs(w, 41)
    ref = oracle_full(w, inputs)
    plain = replay.ShardRun(w, inputs, DEV)
    plain.step()
    scaled_inputs = dict(inputs, d_o=inputs["d_o"] * 64)
    assert torch.equal((scaled_inputs["d_o"].float() / 64).to(torch.bfloat16), inputs["d_o"])
    big = replay.ShardRun(w, scaled_inputs, DEV)
    big.step()
    torch.cuda.synchronize()
    for j in range(len(w.chunks)):
        assert torch.equal(big.dk[j], plain.dk[j] * 64) and torch.equal(big.dv[j], plain.dv[j] * 64)
    assert torch.equal(big.o, plain.o) and torch.equal(big.lse, plain.lse)
    e_plain, _ = check("dq", plain.dq.cpu(), ref["dq"], "bf16")
    e_big, _ = check("dq with residuals everywhere", (big.dq / 64).cpu(), ref["dq"], "bf16")
    frac = float((big.dq / 64 != plain.dq).float().mean())
    print(f"    dq elements changed by the residual path: {100 * frac:.1f} %", flush=True)
    assert frac > 0.5 and e_big <= e_plain


def test_future_chunk_and_merge_outputs():
    dev = torch.device(DEV)
    w = _custom("future", "bf16", 2, 1, 128, 512, [(0, 128)], [[(256, 256)]])
    inputs = wl.make_inputs(w, 3)
    q, d_o = inputs["q"].to(dev), inputs["d_o"].to(dev)
    kc = wl.gather_rows(inputs["k"], w.chunks[0]).to(dev)
    vc = wl.gather_rows(inputs["v"], w.chunks[0]).to(dev)
    desc = hexi.desc_for(q, kc, w.scale)
    o = torch.full((128, 2, 128), 9.0, dtype=torch.float32, device=dev)
    lse = torch.full((2, 128), 9.0, dtype=torch.float32, device=dev)
    hexi.hexi_attn_fwd_chunk(desc, w.q_segs, w.chunks[0], q, kc, vc, o, lse)
    assert torch.all(o == 0) and torch.all(lse == float("-inf"))
    o.fill_(1.5); lse.fill_(0.25)
    hexi.hexi_attn_fwd_chunk(desc, w.q_segs, w.chunks[0], q, kc, vc, o, lse, flags=hexi.HEXI_ACCUMULATE)
    assert torch.all(o == 1.5) and torch.all(lse == 0.25)
    dq = torch.zeros_like(o)
    dk = torch.full((256, 1, 128), 3.0, dtype=torch.float32, device=dev)
    dv = torch.full_like(dk, 3.0)
    delta = torch.zeros_like(lse)
    hexi.hexi_attn_bwd_chunk(desc, w.q_segs, w.chunks[0], q, kc, vc, o, d_o, lse, delta, dq, dk, dv)
    assert torch.all(dk == 0) and torch.all(dv == 0) and torch.all(dq == 0)
    # merge: -inf identities, bf16 and fp32 o_final, against the oracle's merge
    g = torch.Generator().manual_seed(1)
    o_a = torch.randn((300, 3, 128), generator=g); o_b = torch.randn((300, 3, 128), generator=g)
    l_a = torch.randn((3, 300), generator=g) * 4; l_b = torch.randn((3, 300), generator=g) * 4
    l_a[0, :10] = float("-inf"); l_b[1, 5:20] = float("-inf"); l_b[0, :5] = float("-inf")
    o_a[0:10, 0] = 0; o_b[5:20, 1] = 0; o_b[0:5, 0] = 0
    o_ref, l_ref = oracle.merge(to64(o_a), to64(l_a), to64(o_b), to64(l_b))
    for fdt in (None, torch.float32, torch.bfloat16):
        oa, la = o_a.to(dev), l_a.to(dev)
        fin = None if fdt is None else torch.empty((300, 3, 128), dtype=fdt, device=dev)
        hexi.hexi_attn_merge_lse(oa, la, o_b.to(dev), l_b.to(dev), o_final=fin)
        check("merge.o", oa.cpu(), o_ref, "f32")
        check("merge.lse", la.cpu(), l_ref, "f32")
        if fdt is torch.float32:
            assert torch.equal(fin, oa)
        if fdt is torch.bfloat16:
            assert torch.equal(fin, oa.to(torch.bfloat16))


def test_backward_halves_and_dq_reproducible():
    # HEXI_SKIP_DQ / HEXI_SKIP_DKDV run the two halves of the step separately; together they equal the full
    # call.  dq (bf16 path) has a fixed summation order: bit-identical between runs.
    w = wl.config(3, shrink=32)
    inputs = wl.make_inputs(w)
    run = replay.ShardRun(w, inputs, DEV)
    run.step(); torch.cuda.synchronize()
    dq_full = run.dq.clone()
    dk_full = [x.clone() for x in run.dk]
    run.dq.zero_()
    for j, ch in enumerate(w.chunks):
        run.dk[j].fill_(7.0); run.dv[j].fill_(7.0)
        hexi.hexi_attn_bwd_chunk(run.desc[j], w.q_segs, ch, run.q, run.k[j], run.v[j], run.o, run.d_o, run.lse, run.delta,
                                 run.dq, None, None, flags=hexi.HEXI_SKIP_DKDV)
    torch.cuda.synchronize()
    assert torch.equal(run.dq, dq_full)
    assert all(torch.all(x == 7.0) for x in run.dk)
    dq_before = run.dq.clone()
    for j, ch in enumerate(w.chunks):
        hexi.hexi_attn_bwd_chunk(run.desc[j], w.q_segs, ch, run.q, run.k[j], run.v[j], run.o, run.d_o, run.lse, run.delta,
                                 None, run.dk[j], run.dv[j], flags=hexi.HEXI_SKIP_DQ)
    torch.cuda.synchronize()
    assert torch.equal(run.dq, dq_before)
    for a, b in zip(run.dk, dk_full):
        assert torch.allclose(a, b, rtol=1e-4, atol=1e-5)
    with pytest.raises(hexi.HexiError) as e:
        hexi.hexi_attn_bwd_chunk(run.desc[0], w.q_segs, w.chunks[0], run.q, run.k[0], run.v[0], run.o, run.d_o, run.lse,
                                 run.delta, run.dq, run.dk[0], run.dv[0], flags=hexi.HEXI_SKIP_DQ | hexi.HEXI_SKIP_DKDV)
    assert e.value.code == hexi.HEXI_EINVAL


def test_dkdv_reproducible_when_a_workgroup_sums_the_whole_group(force_run_len):
    # whole-group head runs use plain stores and a fixed summation order: dk / dv are bit-identical between runs
    # (runs that split a group add with floating-point atomics, whose order may vary)
    w = wl.config(2, shrink=16)
    inputs = wl.make_inputs(w)
    run = replay.ShardRun(w, inputs, DEV)
    run.forward()
    force_run_len(w.n_q_heads // w.n_kv_heads)
    run.backward(); torch.cuda.synchronize()
    first = [(a.clone(), b.clone()) for a, b in zip(run.dk, run.dv)]
    for a, b in zip(run.dk, run.dv):
        a.fill_(float("nan")); b.fill_(float("nan"))
    run.backward(); torch.cuda.synchronize()
    for (a0, b0), a1, b1 in zip(first, run.dk, run.dv):
        assert torch.equal(a0, a1) and torch.equal(b0, b1)


def test_forward_is_deterministic():
    w = wl.config(3, shrink=32)
    inputs = wl.make_inputs(w)
    run = replay.ShardRun(w, inputs, DEV)
    run.forward(); torch.cuda.synchronize()
    o1, l1 = run.o.clone(), run.lse.clone()
    run.forward(); torch.cuda.synchronize()
    assert torch.equal(o1, run.o) and torch.equal(l1, run.lse)


@pytest.mark.parametrize("lq,lc", [(1, 1), (63, 65), (255, 64), (256, 129), (257, 300), (600, 192), (513, 1)])
def test_workgroup_boundary_sizes(lq, lc):
    # shard / chunk lengths just below, at and above the kernels' workgroup tiles (256 q rows, 128 / 64 keys):
    # one, two and a fraction of a tile, a single row, a single key; two chunks so that the second is diagonal
    l_tot = lc + lq
    q_segs = [(lc, lq)]
    chunks = [[(0, lc)], [(lc, lq)]]
    w = _custom(f"edge_{lq}_{lc}", "bf16", 2, 1, 128, l_tot, q_segs, chunks)
    _run_and_compare(w, seed=lq * 1000 + lc)


@pytest.mark.parametrize("d", [128, 64])
def test_forward_exact_softmax_fallback(d):
    # The fast forward path fixes each row's softmax reference after its first key tile and repeats the
    # workgroup with the exact online softmax when a row's sum leaves [2^-60, 2^60].  Keys beyond the first
    # tile are scaled so that later scores exceed the first tile's maximum by far more than 2^100 (rows 0-255,
    # both wave groups, upward), and a second shard does the reverse (first tile huge, the rest tiny: downward
    # is harmless but must stay exact too).  Everything is compared with the oracle.
    dev = torch.device(DEV)
    g = torch.Generator().manual_seed(99)
    lq, lc, nq = 300, 640, 2
    for first_scale, later_scale in ((1.0, 60.0), (60.0, 0.02)):
        q = (torch.randn((lq, nq, d), generator=g) * 3).to(torch.bfloat16)
        k = torch.randn((lc, 1, d), generator=g)
        k[:64] *= first_scale
        k[64:] *= later_scale
        k = k.to(torch.bfloat16)
        v = torch.randn((lc, 1, d), generator=g).to(torch.bfloat16)
        scale = d ** -0.5
        qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
        o = torch.zeros((lq, nq, d), dtype=torch.float32, device=dev)
        lse = torch.full((nq, lq), float("-inf"), dtype=torch.float32, device=dev)
        q_segs, kv_segs = [(lc, lq)], [(0, lc)]
        hexi.hexi_attn_fwd_chunk(hexi.desc_for(qd, kd, scale), q_segs, kv_segs, qd, kd, vd, o, lse)
        torch.cuda.synchronize()
        o_ref, lse_ref = oracle.attn_fwd(to64(q), np.arange(lc, lc + lq), to64(k), to64(v), np.arange(lc), scale)
        spread = float(np.max(lse_ref) - np.min(lse_ref))
        print(f"  scales {first_scale}/{later_scale}: lse range {np.min(lse_ref):.1f} .. {np.max(lse_ref):.1f}", flush=True)
        assert spread > 50.0     # the case really spans a wide range
        check("o", o.cpu(), o_ref, "bf16")
        check("lse", lse.cpu(), lse_ref, "bf16")     # values in the hundreds, still inside the flat bound


def test_device_share_of_a_scheduled_plan():
    # host scheduler -> shard descriptor -> attention kernels: with 3 heads on two fast + two slow devices the
    # plan is two node groups of uneven length with uneven head counts; one device per group runs its share
    # (its group's block, its head range, which cuts through a GQA group; the ring's blocks in order, the
    # later group's block lying in the first group's future) against the oracle
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from sched_util import cluster_arrays, model_args
    arr = cluster_arrays([("h100", 2), ("a800", 2)])
    plan = hexi.hexi_sched_solve(arr, model_args(l_tot=4096, n_heads=3, hidden=384), token_quantum=64, m2=4, i_max=20)
    print("\nplan:", plan)
    assert plan["groups"] == [[0, 1], [2, 3]] and sum(plan["l_group"]) == 4096 and plan["l_group"][0] != plan["l_group"][1]
    for dev in (1, 2):
        w = wl.from_schedule(plan["groups"], plan["l_group"], plan["n_heads"], dev, head_dim=128, q_per_kv=2)
        assert w.n_q_heads == plan["n_heads"][dev] and len(w.chunks) == 2
        _run_and_compare(w, seed=31 + dev)


def test_measured_compute_rate_feeds_the_scheduler():
    # c_d of the cost model (Eq. 11 convention: 16 * Lq * Lc * n_d * d_h flop per fully visible step) measured on
    # this GPU through the library's own kernels, then used as the compute rate of a homogeneous 8-device plan
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from sched_util import cluster_arrays, model_args
    from paper_2605_07569_amd import calibrate
    c_d = calibrate.measure_c_d(lq=4096, lc=4096, reps=3)
    print(f"\n  measured c_d = {c_d / 1e12:.0f} TFLOP/s (Eq. 11 convention)", flush=True)
    # 14/16 of it is the counted rate on unmasked pairs: between a tenth of and the whole bf16 MFMA roof
    assert 0.25e15 < c_d < 2.9e15
    arr = cluster_arrays([("h100", 8)])
    arr["c"] = np.full(8, c_d)
    model = model_args(l_tot=65536, n_heads=32, hidden=4096)
    plan = hexi.hexi_sched_solve(arr, model, m2=4, i_max=10)
    assert sum(plan["l_group"]) == 65536 and all(sum(plan["n_heads"][d] for d in g) == 32 for g in plan["groups"])
    t_blk, t_non, t_a2a, t_ring, feasible = hexi.hexi_sched_cost(arr, model, plan["groups"], plan["l_group"], plan["s_pre"], plan["n_heads"])
    assert feasible and abs(t_blk - plan["cost"]) <= 1e-12 * t_blk
    # a slower device rate can only raise the modelled ring time
    arr_slow = dict(arr, c=np.full(8, c_d / 4))
    assert hexi.hexi_sched_cost(arr_slow, model, plan["groups"], plan["l_group"], plan["s_pre"], plan["n_heads"])[3] >= t_ring
