"""The library's C++ scheduler and performance model against the Python oracle (oracle/scheduler.py):
cost terms of random valid schedules to 1e-12 relative, feasibility flags equal, and the searched
schedule identical (integers bit-exact, cost to 1e-12).  Host code only: runs without a GPU."""
import time

import numpy as np
import pytest

from oracle import scheduler as S
from paper_2605_07569_amd import hexi
from sched_util import cluster_arrays, model_args


def _oracle_objs(arr, margs):
    return S.Cluster(**arr), S.Model(**margs)


def _random_schedule(rng, n, l_tot, n_heads, q=64):
    k = int(rng.integers(1, n + 1))
    perm = list(range(n))
    cuts = sorted(rng.choice(np.arange(1, n), size=k - 1, replace=False).tolist()) if k > 1 else []
    groups = [perm[a:b] for a, b in zip([0] + cuts, cuts + [n])]
    units = l_tot // q
    lg = rng.multinomial(units - k, np.ones(k) / k) + 1
    l_group = [int(x) * q for x in lg]
    s_pre, nh = [0] * n, [0] * n
    for g, L in zip(groups, l_group):
        parts = rng.multinomial(L // q, np.ones(len(g)) / len(g))
        heads = rng.multinomial(n_heads, rng.dirichlet(np.ones(len(g))))
        for d, p, h in zip(g, parts, heads):
            s_pre[d], nh[d] = int(p) * q, int(h)
    return groups, l_group, s_pre, nh


@pytest.mark.parametrize("nodes,seed", [([("h100", 4), ("a100", 4)], 1), ([("h100", 2), ("a100", 3), ("a800", 2)], 2), ([("a100", 1)], 3)])
def test_cost_terms_match_oracle_on_random_schedules(nodes, seed):
    arr = cluster_arrays(nodes, jitter_seed=seed)
    margs = model_args(l_tot=65536, n_heads=32)
    cl, mo = _oracle_objs(arr, margs)
    rng = np.random.default_rng(seed)
    for _ in range(40):
        groups, l_group, s_pre, nh = _random_schedule(rng, cl.n, margs["l_tot"], margs["n_heads"])
        T = S.Schedule(groups, l_group, s_pre, nh)
        assert S.valid(cl, mo, T)
        got = hexi.hexi_sched_cost(arr, margs, groups, l_group, s_pre, nh)
        want = (S.t_blk(cl, mo, T), max(S.t_nonattn(cl, mo, T, d) for d in range(cl.n)),
                max(S.t_a2a(cl, mo, T, k) for k in range(len(groups))), sum(S.t_step(cl, mo, T, t) for t in range(len(groups))))
        for g, w in zip(got[:4], want):
            assert g == pytest.approx(w, rel=1e-12, abs=0.0)
        assert got[4] == S.feasible(cl, mo, T)


def test_memory_flag_and_constraint_errors():
    arr = cluster_arrays([("a100", 2)])
    margs = model_args(l_tot=4096)
    ok = hexi.hexi_sched_cost(arr, margs, [[0, 1]], [4096], [2048, 2048], [16, 16])
    assert ok[4] is True
    tight = dict(arr, m=[arr["m_static"][0] + 67108863.0, 80e9])          # one byte short of Mem_act (App. A.2)
    assert hexi.hexi_sched_cost(tight, margs, [[0, 1]], [4096], [2048, 2048], [16, 16])[4] is False
    for bad in (([[0, 1]], [4096], [2048, 2047], [16, 16]),                 # shards do not sum to L_k
                ([[0, 1]], [4096], [2048, 2048], [16, 15]),                 # heads do not cover N
                ([[0], [1]], [2048, 1024], [2048, 1024], [32, 32])):        # lengths do not sum to L_tot
        with pytest.raises(RuntimeError):
            hexi.hexi_sched_cost(arr, margs, *bad)
    with pytest.raises(RuntimeError):                                       # nothing fits: no feasible schedule
        hexi.hexi_sched_solve(dict(arr, m=[arr["m_static"][0] + 1.0] * 2), margs)
    assert "memory filter" in hexi.load().hexi_last_error().decode()


@pytest.mark.parametrize("nodes,margs,opts", [
    ([("h100", 2), ("a100", 2)], model_args(l_tot=16384, n_heads=8, hidden=1024), dict(m1=8, m2=4, i_max=20)),
    ([("h100", 4), ("a100", 4)], model_args(l_tot=131072, n_heads=32), dict()),
    ([("h100", 2), ("a100", 2), ("a800", 2)], model_args(l_tot=32768, n_heads=40, hidden=5120), dict(m2=6, i_max=30)),
])
def test_solve_matches_oracle_exactly(nodes, margs, opts):
    arr = cluster_arrays(nodes, jitter_seed=7)
    cl, mo = _oracle_objs(arr, margs)
    T, C = S.solve(cl, mo, **opts)
    got = hexi.hexi_sched_solve(arr, margs, **opts)
    assert got["groups"] == T.groups
    assert got["l_group"] == T.l_group and got["s_pre"] == T.s_pre and got["n_heads"] == T.n_heads
    assert got["cost"] == pytest.approx(C, rel=1e-12)
    # and the library scores its own answer the same way
    assert hexi.hexi_sched_cost(arr, margs, got["groups"], got["l_group"], got["s_pre"], got["n_heads"])[0] == pytest.approx(got["cost"], rel=1e-12)


def test_solve_beats_symmetric_baselines_and_scales():
    # the paper's Setting 3 (8 H100 + 8 A100, Sec. 5.2): not worse than Ring / Ulysses / USP by construction
    arr = cluster_arrays([("h100", 8), ("a100", 8)])
    margs = model_args(l_tot=65536, n_heads=32)
    t0 = time.perf_counter()
    got = hexi.hexi_sched_solve(arr, margs)
    dt = time.perf_counter() - t0
    n = 16
    ring = hexi.hexi_sched_cost(arr, margs, [[d] for d in range(n)], [4096] * n, [4096] * n, [32] * n)[0]
    ulysses = hexi.hexi_sched_cost(arr, margs, [list(range(n))], [65536], [4096] * n, [2] * n)[0]
    usp = hexi.hexi_sched_cost(arr, margs, [list(range(8)), list(range(8, 16))], [32768, 32768], [4096] * n, [4] * n)[0]
    assert got["cost"] <= min(ring, ulysses, usp)
    assert sum(got["l_group"]) == 65536 and all(sum(got["n_heads"][d] for d in g) == 32 for g in got["groups"])
    print(f"\\n16 devices: cost {got['cost']:.4f} s vs ring {ring:.4f} ulysses {ulysses:.4f} usp {usp:.4f}; solved in {dt:.2f} s; groups {got['groups']}")
    assert dt < 60.0
