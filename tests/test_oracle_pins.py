"""Pins for the fp64 CPU oracle: closed forms, invariants, finite differences, brute force.

The paper gives no worked numerical example of attention, so every pin comes from the mathematics of
the definition it presupposes.  Each test is chosen so that a plausible mistake in the oracle (a
dropped term, a wrong sign, an off-by-one in the causal mask, a transposed operand, a wrong head map)
fails it.  None of these tests touches the HIP library.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_07569_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _problem(rng, q_segs, l_tot, nq, nkv, d):
    q_pos = oracle.positions(q_segs)
    kv_pos = np.arange(l_tot, dtype=np.int64)
    q = rng.standard_normal((len(q_pos), nq, d))
    k = rng.standard_normal((l_tot, nkv, d))
    v = rng.standard_normal((l_tot, nkv, d))
    d_o = rng.standard_normal((len(q_pos), nq, d))
    return q, q_pos, k, v, kv_pos, d_o


def test_golden_two_key_example():
    g = json.load(open(os.path.join(GOLD, "two_key_softmax.json")))
    q, k, v, d_o = (np.array(g[n]) for n in ("q", "k", "v", "d_o"))
    c = g["case_sees_both"]
    o, lse = oracle.attn_fwd(q, c["q_pos"], k, v, g["kv_pos"], g["scale"])
    assert abs(o[0, 0, 0] - c["o"]) < 1e-14 and abs(lse[0, 0] - c["lse"]) < 1e-14
    r = oracle.attn_bwd(q, c["q_pos"], k, v, g["kv_pos"], d_o, g["scale"])
    assert abs(r["delta"][0, 0] - c["delta"]) < 1e-14
    assert abs(r["dq"][0, 0, 0] - c["dq"]) < 1e-14
    np.testing.assert_allclose(r["dv"][:, 0, 0], c["dv"], atol=1e-14)
    np.testing.assert_allclose(r["dk"][:, 0, 0], np.array(c["ds"]) * math.log(2.0), atol=1e-14)
    c = g["case_sees_first_only"]
    o, lse = oracle.attn_fwd(q, c["q_pos"], k, v, g["kv_pos"], g["scale"])
    assert o[0, 0, 0] == c["o"] and lse[0, 0] == c["lse"]
    r = oracle.attn_bwd(q, c["q_pos"], k, v, g["kv_pos"], d_o, g["scale"])
    assert r["dq"][0, 0, 0] == c["dq"]
    np.testing.assert_allclose(r["dv"][:, 0, 0], c["dv"], atol=1e-15)
    assert np.all(r["dk"] == 0.0)


def test_p1_probability_rows_sum_to_one():
    rng = np.random.default_rng(1)
    q, q_pos, k, v, kv_pos, _ = _problem(rng, [(3, 5), (20, 7)], 40, 4, 2, 8)
    o, _ = oracle.attn_fwd(q, q_pos, k, np.ones_like(v), kv_pos, 0.35)
    assert np.max(np.abs(o - 1.0)) < 1e-12


def test_p2_merge_over_any_partition_equals_one_shot():
    rng = np.random.default_rng(2)
    q, q_pos, k, v, kv_pos, _ = _problem(rng, [(2, 6), (30, 9)], 48, 6, 3, 8)
    scale = 0.4
    o_ref, lse_ref = oracle.attn_fwd(q, q_pos, k, v, kv_pos, scale)
    for trial in range(6):
        n_cuts = [1, 3, 7, 12, 47, 5][trial]
        cuts = np.sort(rng.choice(np.arange(1, 48), size=n_cuts, replace=False))
        edges = [0] + cuts.tolist() + [48]
        parts = [(a, b) for a, b in zip(edges[:-1], edges[1:])] + [(17, 17)]  # plus an empty part
        order = rng.permutation(len(parts))
        o_acc = np.zeros_like(o_ref)
        lse_acc = np.full_like(lse_ref, -np.inf)
        for pi in order:
            a, b = parts[pi]
            o_p, lse_p = oracle.attn_fwd(q, q_pos, k[a:b], v[a:b], kv_pos[a:b], scale)
            assert not np.any(np.isnan(o_p)) and not np.any(np.isnan(lse_p))
            o_acc, lse_acc = oracle.merge(o_acc, lse_acc, o_p, lse_p)
        np.testing.assert_allclose(o_acc, o_ref, rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse_acc, lse_ref, rtol=0, atol=1e-12)


def test_p2b_merge_identities_with_minus_inf():
    rng = np.random.default_rng(22)
    o_a = rng.standard_normal((5, 2, 4))
    lse_a = rng.standard_normal((2, 5))
    zero, ninf = np.zeros_like(o_a), np.full_like(lse_a, -np.inf)
    o, lse = oracle.merge(o_a, lse_a, zero, ninf)
    assert np.array_equal(o, o_a) and np.array_equal(lse, lse_a)
    o, lse = oracle.merge(zero, ninf, o_a, lse_a)
    assert np.array_equal(o, o_a) and np.array_equal(lse, lse_a)
    o, lse = oracle.merge(zero, ninf, zero, ninf)
    assert np.all(o == 0) and np.all(lse == -np.inf)
    # equal LSEs: plain average, LSE + ln 2
    o_b = rng.standard_normal((5, 2, 4))
    o, lse = oracle.merge(o_a, lse_a, o_b, lse_a)
    np.testing.assert_allclose(o, 0.5 * (o_a + o_b), atol=1e-15)
    np.testing.assert_allclose(lse, lse_a + math.log(2.0), atol=1e-15)


def test_p3_token_zero_sees_only_itself():
    rng = np.random.default_rng(3)
    q, q_pos, k, v, kv_pos, d_o = _problem(rng, [(0, 4), (11, 3)], 16, 4, 2, 8)
    scale = 0.3
    o, lse = oracle.attn_fwd(q, q_pos, k, v, kv_pos, scale)
    for h in range(4):
        g = h // 2
        np.testing.assert_allclose(o[0, h], v[0, g], atol=1e-15)
        assert abs(lse[h, 0] - scale * float(q[0, h] @ k[0, g])) < 1e-14
    # a shard entirely before the chunk: nothing visible
    o, lse = oracle.attn_fwd(q, q_pos, k[12:], v[12:], kv_pos[12:] + 100, scale)
    assert np.all(o == 0) and np.all(lse == -np.inf)


def test_p4_gradients_match_finite_differences():
    rng = np.random.default_rng(4)
    q, q_pos, k, v, kv_pos, d_o = _problem(rng, [(3, 3), (9, 3)], 12, 4, 2, 4)
    scale = 0.45
    kv_of_q = [0, 1, 1, 0]  # a non-default head map

    def loss(q_, k_, v_):
        o, _ = oracle.attn_fwd(q_, q_pos, k_, v_, kv_pos, scale, kv_of_q)
        return float(np.sum(o * d_o))

    r = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, scale, kv_of_q)
    eps = 1e-6
    for name, x, grad in (("dq", q, r["dq"]), ("dk", k, r["dk"]), ("dv", v, r["dv"])):
        fd = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = dict(q_=q, k_=k, v_=v)
            args_m = dict(args_p)
            key = {"dq": "q_", "dk": "k_", "dv": "v_"}[name]
            args_p[key], args_m[key] = xp, xm
            fd[idx] = (loss(**args_p) - loss(**args_m)) / (2 * eps)
        err = np.max(np.abs(fd - grad)) / max(1e-30, np.max(np.abs(grad)))
        assert err < 1e-7, (name, err)


@pytest.mark.parametrize("q_segs,l_tot", [([(5, 9)], 20), ([(0, 4), (28, 4)], 32), ([(7, 1), (9, 2), (30, 5)], 40)])
def test_p5_zero_query_closed_form(q_segs, l_tot):
    rng = np.random.default_rng(5)
    q, q_pos, k, v, kv_pos, d_o = _problem(rng, q_segs, l_tot, 4, 2, 6)
    q[:] = 0.0
    r = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, 0.5)
    o, lse = oracle.attn_fwd(q, q_pos, k, v, kv_pos, 0.5)
    csum = np.cumsum(v, axis=0)
    for i, p in enumerate(q_pos):
        assert np.max(np.abs(lse[:, i] - math.log(p + 1))) < 1e-13
        for h in range(4):
            np.testing.assert_allclose(o[i, h], csum[p, h // 2] / (p + 1), atol=1e-13)
    dv_ref = np.zeros_like(v)
    for j in range(l_tot):
        for i, p in enumerate(q_pos):
            if p >= j:
                for h in range(4):
                    dv_ref[j, h // 2] += d_o[i, h] / (p + 1)
    np.testing.assert_allclose(r["dv"], dv_ref, atol=1e-13)
    np.testing.assert_allclose(r["lse"], lse, atol=1e-14)


def test_p6_backward_row_and_column_sums():
    rng = np.random.default_rng(6)
    q, q_pos, k, v, kv_pos, d_o = _problem(rng, [(4, 10)], 24, 6, 2, 8)
    r = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, 0.3)
    # sum_j dV_j = sum over the group's heads and rows of dO (every row's probabilities sum to 1)
    for g in range(2):
        np.testing.assert_allclose(r["dv"][:, g].sum(0), d_o[:, 3 * g:3 * g + 3].sum((0, 1)), atol=1e-12)
    # identical keys: dQ_i = scale * (sum_j dS_ij) * c = 0 because the rows of dS sum to zero
    k_same = np.broadcast_to(rng.standard_normal((1, 2, 8)), k.shape).copy()
    r2 = oracle.attn_bwd(q, q_pos, k_same, v, kv_pos, d_o, 0.3)
    assert np.max(np.abs(r2["dq"])) < 1e-13
    # delta agrees with its standalone definition on the forward output
    o, _ = oracle.attn_fwd(q, q_pos, k, v, kv_pos, 0.3)
    np.testing.assert_allclose(r["delta"], oracle.delta(o, d_o), atol=1e-13)
    np.testing.assert_allclose(oracle.delta(o, d_o), np.einsum("ihc,ihc->hi", o, d_o), atol=1e-13)


def test_p7_q_dq_equals_k_dk():
    rng = np.random.default_rng(7)
    q, q_pos, k, v, kv_pos, d_o = _problem(rng, [(2, 5), (15, 6)], 24, 4, 2, 8)
    r = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, 0.37)
    lhs, rhs = float(np.sum(q * r["dq"])), float(np.sum(k * r["dk"]))
    assert abs(lhs - rhs) < 1e-12 * max(1.0, abs(lhs))
    assert abs(lhs) > 1e-3  # not trivially zero


def test_p8_key_shift_invariance():
    rng = np.random.default_rng(8)
    q, q_pos, k, v, kv_pos, d_o = _problem(rng, [(6, 8)], 16, 4, 4, 8)
    c = rng.standard_normal((1, 1, 8))
    scale = 0.25
    a = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, scale)
    b = oracle.attn_bwd(q, q_pos, k + c, v, kv_pos, d_o, scale)
    oa, _ = oracle.attn_fwd(q, q_pos, k, v, kv_pos, scale)
    ob, _ = oracle.attn_fwd(q, q_pos, k + c, v, kv_pos, scale)
    np.testing.assert_allclose(oa, ob, atol=1e-12)
    np.testing.assert_allclose(a["dv"], b["dv"], atol=1e-12)
    shift = scale * np.einsum("ihc,c->hi", q, c[0, 0])
    np.testing.assert_allclose(b["lse"] - a["lse"], shift, atol=1e-12)


def test_p9_gqa_equals_mha_on_repeated_kv():
    rng = np.random.default_rng(9)
    q, q_pos, k, v, kv_pos, d_o = _problem(rng, [(3, 7)], 12, 6, 2, 4)
    a = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, 0.5)
    k_rep, v_rep = np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1)
    b = oracle.attn_bwd(q, q_pos, k_rep, v_rep, kv_pos, d_o, 0.5)
    np.testing.assert_allclose(a["dq"], b["dq"], atol=1e-13)
    np.testing.assert_allclose(a["dk"], b["dk"].reshape(12, 2, 3, 4).sum(2), atol=1e-13)
    np.testing.assert_allclose(a["dv"], b["dv"].reshape(12, 2, 3, 4).sum(2), atol=1e-13)
    # an explicit, permuted head map is honoured
    perm = [1, 0, 1, 0, 0, 1]
    c = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, 0.5, perm)
    for h, g in enumerate(perm):
        e = oracle.attn_bwd(q[:, h:h + 1], q_pos, k[:, g:g + 1], v[:, g:g + 1], kv_pos, d_o[:, h:h + 1], 0.5)
        np.testing.assert_allclose(c["dq"][:, h], e["dq"][:, 0], atol=1e-13)


def test_p10_whole_sequence_matches_library_sdpa_and_autograd():
    rng = np.random.default_rng(10)
    L, nq, nkv, d = 24, 4, 2, 8
    q, q_pos, k, v, kv_pos, d_o = _problem(rng, [(0, L)], L, nq, nkv, d)
    scale = 1.0 / math.sqrt(d)
    tq = torch.tensor(q.transpose(1, 0, 2), requires_grad=True)              # [h, L, d]
    tk = torch.tensor(k.transpose(1, 0, 2), requires_grad=True)
    tv = torch.tensor(v.transpose(1, 0, 2), requires_grad=True)
    out = torch.nn.functional.scaled_dot_product_attention(
        tq, tk.repeat_interleave(2, 0), tv.repeat_interleave(2, 0), is_causal=True, scale=scale)
    (out * torch.tensor(d_o.transpose(1, 0, 2))).sum().backward()
    r = oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, scale)
    o, _ = oracle.attn_fwd(q, q_pos, k, v, kv_pos, scale)
    np.testing.assert_allclose(o, out.detach().numpy().transpose(1, 0, 2), atol=1e-12)
    np.testing.assert_allclose(r["dq"], tq.grad.numpy().transpose(1, 0, 2), atol=1e-12)
    np.testing.assert_allclose(r["dk"], tk.grad.numpy().transpose(1, 0, 2), atol=1e-12)
    np.testing.assert_allclose(r["dv"], tv.grad.numpy().transpose(1, 0, 2), atol=1e-12)


def _closed_form_pairs(q_segs, kv_segs):
    """Pairs (i, j) with pos(j) <= pos(i): per q position p and kv segment [s, s+n): clamp(p-s+1, 0, n)."""
    total = 0
    for qs, qn in q_segs:
        for s, n in kv_segs:
            for p in (range(qs, qs + qn) if qn <= 4096 else ()):
                total += min(max(p - s + 1, 0), n)
            if qn > 4096:  # arithmetic-series form for long segments
                lo, hi = qs, qs + qn - 1
                a = max(lo, s)                # first p with p - s + 1 >= 1
                b = min(hi, s + n - 1)        # last p still inside the ramp
                if a <= b:
                    total += (a - s + 1 + b - s + 1) * (b - a + 1) // 2
                if hi >= s + n:
                    total += n * (hi - max(lo, s + n) + 1)
    return total


def test_p11_pair_counts_closed_form_and_bruteforce():
    gold = json.load(open(os.path.join(GOLD, "config_pair_counts.json")))["n_pairs"]
    for idx in range(1, 6):
        w = wl.config(idx)
        total = sum(_closed_form_pairs(w.q_segs, ch) for ch in w.chunks)
        assert total == gold[str(idx)], (idx, total)
        assert sum(n for ch in w.chunks for _, n in ch) == w.l_tot
    # brute force on shrunken configs and ragged random segment lists agrees with the closed form
    for idx, shrink in ((1, 8), (2, 128), (3, 256), (4, 256), (5, 512)):
        w = wl.config(idx, shrink=shrink)
        for ch in w.chunks:
            cls, n = oracle.mask_bruteforce(oracle.positions(w.q_segs), oracle.positions(ch), 16, 16)
            assert n == _closed_form_pairs(w.q_segs, ch)
    rng = np.random.default_rng(11)
    for _ in range(10):
        def segs(n_seg):
            lens = rng.integers(1, 60, n_seg)
            gaps = rng.integers(0, 40, n_seg)
            out, cur = [], 0
            for ln, gp in zip(lens, gaps):
                cur += int(gp)
                out.append((cur, int(ln)))
                cur += int(ln)
            return out
        qs, ks = segs(rng.integers(1, 5)), segs(rng.integers(1, 5))
        qp, kp = oracle.positions(qs), oracle.positions(ks)
        cls, n = oracle.mask_bruteforce(qp, kp, 7, 5)
        vis = kp[None, :] <= qp[:, None]
        assert n == int(vis.sum()) == _closed_form_pairs(qs, ks)
        for tm in range(cls.shape[0]):
            for tn in range(cls.shape[1]):
                blk = vis[tm * 7:(tm + 1) * 7, tn * 5:(tn + 1) * 5]
                want = 0 if not blk.any() else (1 if blk.all() else 2)
                assert cls[tm, tn] == want


def test_p12_zigzag_chunks_are_half_visible():
    for idx, r_own in ((2, 0), (4, 3)):
        w = wl.config(idx)
        lq = w.lq
        blk = lq // 2
        for j, ch in enumerate(w.chunks):
            n = _closed_form_pairs(w.q_segs, ch)
            lc = sum(x for _, x in ch)
            half = lq * lc // 2
            if j == r_own:
                # own chunk: the two diagonal blocks each add their diagonal: 2 * blk/2 pairs over half
                assert n == half + blk
            else:
                assert n == half
    # positions() packs segments in order
    assert oracle.positions([(5, 2), (9, 3)]).tolist() == [5, 6, 9, 10, 11]
