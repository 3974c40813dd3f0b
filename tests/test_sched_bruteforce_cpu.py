"""The scheduler's search (Sec. 4.3; oracle/scheduler.py and the library's hexi_sched_solve) against an exhaustive
enumeration of the schedule space of Sec. 4.1 on clusters small enough to enumerate (oracle/sched_bruteforce.py):
a search can never beat the true optimum, and on these cases the three stages do reach it."""
import math

import pytest

from oracle import sched_bruteforce as BF
from oracle import scheduler as S
from paper_2605_07569_amd import hexi
from sched_util import cluster_arrays, model_args


def test_enumerator_counts_match_closed_forms():
    # set partitions: Bell numbers; blocks ordered by smallest element
    assert [sum(1 for _ in BF.set_partitions(list(range(n)))) for n in range(1, 6)] == [1, 2, 5, 15, 52]
    assert sorted(BF.set_partitions([0, 1, 2])) == sorted([[[0], [1], [2]], [[0, 1], [2]], [[0], [1, 2]], [[0, 2], [1]], [[0, 1, 2]]])
    # compositions of t into k parts >= m: C(t - k m + k - 1, k - 1)
    for t, k, m in ((8, 3, 0), (8, 3, 1), (4, 2, 1), (5, 1, 0), (3, 4, 1)):
        got = list(BF.compositions(t, k, m))
        assert len(got) == (math.comb(t - k * m + k - 1, k - 1) if t >= k * m else 0)
        assert all(sum(c) == t and min(c) >= m for c in got) and len(set(got)) == len(got)
    # two devices, U quanta, N heads: one group: (U + 1)(N + 1) schedules; two groups: U - 1 (each holds all heads)
    arr = cluster_arrays([("h100", 1), ("a100", 1)])
    cl, mo = S.Cluster(**arr), S.Model(**model_args(l_tot=512, n_heads=4, hidden=256, head_dim=64))
    all_s = list(BF.all_schedules(cl, mo, 64))
    assert len(all_s) == 9 * 5 + 7 and all(S.valid(cl, mo, T) for T in all_s)
    assert len({T.key() for T in all_s}) == len(all_s)


CASES = [([("h100", 1), ("a100", 1)], 512, 4), ([("h100", 2), ("a100", 1)], 512, 4),
         ([("h100", 2), ("a100", 2)], 384, 4), ([("h100", 1), ("a100", 2), ("a800", 1)], 384, 3),
         ([("a100", 3)], 512, 5)]


@pytest.mark.parametrize("nodes,l_tot,n_heads", CASES)
def test_search_never_beats_and_here_reaches_the_exhaustive_optimum(nodes, l_tot, n_heads):
    arr = cluster_arrays(nodes)
    margs = model_args(l_tot=l_tot, n_heads=n_heads, hidden=256, head_dim=64)
    cl, mo = S.Cluster(**arr), S.Model(**margs)
    best, best_c, n_all, n_ok = BF.optimum(cl, mo, 64)
    assert n_ok == n_all and S.valid(cl, mo, best)
    T, C = S.solve(cl, mo, q=64, move_tokens=64)
    assert S.valid(cl, mo, T) and S.feasible(cl, mo, T) and C == S.t_blk(cl, mo, T)
    assert C >= best_c * (1 - 1e-12)
    assert C == pytest.approx(best_c, rel=1e-12)
    got = hexi.hexi_sched_solve(arr, margs, token_quantum=64, move_tokens=64)
    assert got["cost"] == pytest.approx(best_c, rel=1e-12)


def test_search_against_the_optimum_under_a_binding_memory_filter():
    # device 2's activation budget admits little: the optimum gives it a short block; the search must stay feasible and
    # cannot be better than the feasible optimum
    arr = cluster_arrays([("h100", 2), ("a100", 1)])
    margs = model_args(l_tot=512, n_heads=4, hidden=256, head_dim=64)
    arr["m"][2] = arr["m_static"][2] + 2.0 * (2.0 * 128 * 256 + 2.0 * 128 * 4 * 64) + 1.0     # Mem_act of s = L = 128, all heads
    cl, mo = S.Cluster(**arr), S.Model(**margs)
    best, best_c, n_all, n_ok = BF.optimum(cl, mo, 64)
    assert 0 < n_ok < n_all
    T, C = S.solve(cl, mo, q=64, move_tokens=64)
    assert S.feasible(cl, mo, T) and C >= best_c * (1 - 1e-12)
    got = hexi.hexi_sched_solve(arr, margs, token_quantum=64, move_tokens=64)
    assert got["cost"] >= best_c * (1 - 1e-12)
    assert hexi.hexi_sched_cost(arr, margs, got["groups"], got["l_group"], got["s_pre"], got["n_heads"])[4] is True
    print(f"\n  feasible optimum {best_c:.6e}, oracle search {C:.6e}, library search {got['cost']:.6e} ({n_ok} of {n_all} schedules fit)")
