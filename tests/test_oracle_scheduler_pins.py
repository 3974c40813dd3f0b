"""Pins of the scheduler / performance-model oracle (oracle/scheduler.py): hand-worked numbers, closed
forms of the symmetric baselines, scaling and monotonicity invariants, structural constraints."""
import math

import pytest

from oracle import scheduler as S
from sched_util import cluster_arrays, model_args


def _cluster(**kw):
    return S.Cluster(**kw)


def _two_device_cluster():
    # round numbers: c = 1e12 FLOP/s, b = 1e11 B/s, links 1e9 B/s with 1 ms startup
    n = 2
    bw = [[1e30, 1e9], [1e9, 1e30]]
    al = [[0.0, 1e-3], [1e-3, 0.0]]
    return S.Cluster([1e12, 1e12], [1e11, 1e11], [1e12, 1e12], [0.0, 0.0], al, bw)


def test_hand_worked_single_group():
    """App. A.3-A.4 with B = 1, H = 1000, d_h = 100, N = 4, P = 2, L_tot = 2000; one group of two devices,
    s = (1000, 1000), n = (2, 2).  By hand:
      F_nonattn = 72 * 1000 * 1000^2 = 7.2e10 -> 0.072 s;  V_nonattn = 40 * 1000 * 1000 * 2 = 8e7 -> 8e-4 s  => 0.072
      V(d->j) = 3 * 1000 * (2 * 100) * 2 = 1.2e6 B -> 1e-3 + 1.2e-3 = 2.2e-3;  T_A2A = 4 * 2.2e-3 = 8.8e-3
      F_step(t=0) = 16 * 2000 * 2000 * (2 * 100) = 1.28e10 -> 0.0128 s (one step, local)
      T_blk = 0.072 + 0.0088 + 0.0128 = 0.0936
      Mem_act = 1 * 2 * (2 * 1000 * 1000 + 2 * 2000 * 200) = 5.6e6 bytes"""
    cl, mo = _two_device_cluster(), S.Model(2000, 1, 1000, 100, 4, 2)
    T = S.Schedule([[0, 1]], [2000], [1000, 1000], [2, 2])
    assert S.valid(cl, mo, T)
    assert S.t_nonattn(cl, mo, T, 0) == pytest.approx(0.072, rel=1e-12)
    assert S.t_a2a(cl, mo, T, 0) == pytest.approx(8.8e-3, rel=1e-12)
    assert S.t_step(cl, mo, T, 0) == pytest.approx(0.0128, rel=1e-12)
    assert S.t_blk(cl, mo, T) == pytest.approx(0.0936, rel=1e-12)
    assert S.mem_act(cl, mo, T, 0, 0) == pytest.approx(5.6e6, rel=1e-12)


def test_hand_worked_two_groups_ring():
    """Same devices as two groups of one (pure ring), L = (1000, 1000), all 4 heads each.  By hand:
      no A2A partner -> T_A2A = 0;  T_nonattn = 0.072
      F_step = 16 * 1000 * 1000 * 400 = 6.4e9 -> 6.4e-3 s for both steps
      Msg = 4 * 1000 * 400 * 2 = 3.2e6 B -> 1e-3 + 3.2e-3 = 4.2e-3 < 6.4e-3, so step 1 is compute-bound
      T_blk = 0.072 + 0 + 2 * 6.4e-3 = 0.0848;  with links of 1e8 B/s the remote step costs 1e-3 + 3.2e-2 = 0.033"""
    cl, mo = _two_device_cluster(), S.Model(2000, 1, 1000, 100, 4, 2)
    T = S.Schedule([[0], [1]], [1000, 1000], [1000, 1000], [4, 4])
    assert S.valid(cl, mo, T)
    assert S.t_a2a(cl, mo, T, 0) == 0.0 and S.t_a2a(cl, mo, T, 1) == 0.0
    assert S.t_step(cl, mo, T, 0) == pytest.approx(6.4e-3, rel=1e-12)
    assert S.t_step(cl, mo, T, 1) == pytest.approx(6.4e-3, rel=1e-12)
    assert S.t_blk(cl, mo, T) == pytest.approx(0.0848, rel=1e-12)
    cl.bw = [[1e30, 1e8], [1e8, 1e30]]
    assert S.t_step(cl, mo, T, 1) == pytest.approx(0.033, rel=1e-12)


def test_overlapping_head_ranges_split_the_message():
    # group 0 = {0, 1} with heads (3, 1), group 1 = {2} with all 4: device 2 receives 3/4 of its message from
    # device 0 and 1/4 from device 1 in parallel; the slower of the two transfers decides (reading r3)
    n = 3
    bw = [[1e30, 1e9, 1e9], [1e9, 1e30, 1e8], [1e9, 1e8, 1e30]]
    al = [[0.0] * n for _ in range(n)]
    cl = S.Cluster([1e15] * n, [1e15] * n, [1e15] * n, [0.0] * n, al, bw)
    mo = S.Model(3000, 1, 1000, 100, 4, 2)
    T = S.Schedule([[0, 1], [2]], [2000, 1000], [1000, 1000, 1000], [3, 1, 4])
    # step 1, device 2: Msg = 4 * 2000 * 400 * 2 = 6.4e6 B; from 0: 4.8e6 / 1e9 = 4.8e-3; from 1: 1.6e6 / 1e8 = 1.6e-2
    # device 0 (3 heads) receives from device 2: 4 * 1000 * 300 * 2 = 2.4e6 / 1e9 = 2.4e-3; device 1: 8e5 / 1e8 = 8e-3
    assert S.t_step(cl, mo, T, 1) == pytest.approx(1.6e-2, rel=1e-9)


def test_symmetric_ring_closed_form_and_scaling():
    arr = cluster_arrays([("a100", 4)])
    cl, mo = _cluster(**arr), S.Model(**{**model_args(l_tot=32768), "gamma_act": 2.0})
    n, L = 4, 32768 // 4
    T = S.Schedule([[d] for d in range(n)], [L] * n, [L] * n, [mo.N] * n)
    c, b, bw, al = arr["c"][0], arr["b"][0], arr["bw"][0][1], arr["alpha"][0][1]
    nonattn = max(72.0 * L * mo.H ** 2 / c, 40.0 * L * mo.H * 2 / b)
    comp = 16.0 * L * L * mo.N * mo.d_h / c
    comm = al + 4.0 * L * mo.N * mo.d_h * 2 / bw
    assert S.t_blk(cl, mo, T) == pytest.approx(nonattn + comp + 3 * max(comp, comm), rel=1e-12)
    # all rates x2 and all startup latencies / 2  =>  every term halves
    fast = _cluster(c=[2 * x for x in arr["c"]], b=[2 * x for x in arr["b"]], m=arr["m"], m_static=arr["m_static"],
                    alpha=[[a / 2 for a in r] for r in arr["alpha"]], bw=[[2 * x for x in r] for r in arr["bw"]])
    assert S.t_blk(fast, mo, T) == pytest.approx(S.t_blk(cl, mo, T) / 2, rel=1e-12)


def test_memory_filter_and_validity():
    arr = cluster_arrays([("a100", 2)])
    cl, mo = _cluster(**arr), S.Model(**model_args(l_tot=4096))
    T = S.Schedule([[0, 1]], [4096], [2048, 2048], [16, 16])
    assert S.valid(cl, mo, T) and S.feasible(cl, mo, T)
    # 1 * 2 * (2 * 2048 * 4096 + 2 * 4096 * 16 * 128) = 67 108 864 bytes per device (App. A.2)
    assert S.mem_act(cl, mo, T, 0, 0) == 67108864.0
    cl.m = [cl.m_static[0] + 67108863.0, 80e9]
    assert not S.feasible(cl, mo, T)
    assert not S.valid(cl, mo, S.Schedule([[0, 1]], [4096], [2048, 2047], [16, 16]))     # shards do not sum to L_k
    assert not S.valid(cl, mo, S.Schedule([[0, 1]], [4096], [2048, 2048], [16, 15]))     # heads do not cover N
    assert not S.valid(cl, mo, S.Schedule([[0], [1]], [2048, 2048], [2048, 2048], [16, 16]))   # each group needs all heads


def test_largest_remainder():
    assert S.largest_remainder(10, [1, 1, 1]) == [4, 3, 3]
    assert S.largest_remainder(640, [3, 1], 64) == [512, 128]
    assert sum(S.largest_remainder(131072, [989.0, 312.0, 312.0, 17.0], 64)) == 131072
    assert all(x % 64 == 0 for x in S.largest_remainder(131072, [989.0, 312.0, 312.0, 17.0], 64))


def test_partitions_contain_baselines_and_node_groups():
    arr = cluster_arrays([("h100", 4), ("a100", 4)])
    parts = S.partition_topology(_cluster(**arr))
    keys = [tuple(tuple(g) for g in p) for p in parts]
    assert tuple((d,) for d in range(8)) in keys                       # Ring
    assert (tuple(range(8)),) in keys                                  # Ulysses
    assert ((0, 1, 2, 3), (4, 5, 6, 7)) in keys                        # USP 2 x 4 = the node-aligned grouping
    assert ((0, 1), (2, 3), (4, 5), (6, 7)) in keys                    # USP 4 x 2
    assert ((0, 1, 2, 3), (4,), (5,), (6,), (7,)) in keys              # agglomeration level at 450 GB/s
    # a 12x slower fabric is a gap: the agglomeration does not merge across it on its own
    only_agglo = [k for k in keys if k not in (tuple((d,) for d in range(8)), (tuple(range(8)),))]
    assert all(max(len(g) for g in k) <= 4 for k in only_agglo)


def test_solve_returns_valid_feasible_schedule_not_worse_than_baselines():
    arr = cluster_arrays([("h100", 2), ("a100", 2)])
    cl, mo = _cluster(**arr), S.Model(**model_args(l_tot=16384, n_heads=8, hidden=1024))
    T, C = S.solve(cl, mo, m1=8, m2=4, i_max=20)
    assert S.valid(cl, mo, T) and S.feasible(cl, mo, T)
    assert C == S.t_blk(cl, mo, T)
    n = 4
    ring = S.Schedule([[d] for d in range(n)], [4096] * n, [4096] * n, [8] * n)
    ulysses = S.Schedule([list(range(n))], [16384], [4096] * n, [2] * n)
    usp = S.Schedule([[0, 1], [2, 3]], [8192, 8192], [4096] * n, [4, 4, 4, 4])
    for base in (ring, ulysses, usp):
        assert S.valid(cl, mo, base)
        assert C <= S.t_blk(cl, mo, base)
    # the faster devices never end up with less attention work than the slower ones of the same group
    for g in T.groups:
        for a in g:
            for b in g:
                if cl.c[a] > cl.c[b]:
                    assert T.n_heads[a] >= T.n_heads[b]


def test_faster_link_or_device_never_hurts_a_fixed_schedule():
    arr = cluster_arrays([("h100", 2), ("a800", 2)], jitter_seed=5)
    cl, mo = _cluster(**arr), S.Model(**model_args(l_tot=8192, n_heads=8))
    T = S.Schedule([[0, 1], [2, 3]], [5120, 3072], [2560, 2560, 1536, 1536], [5, 3, 4, 4])
    base = S.t_blk(cl, mo, T)
    cl.bw[2][3] *= 3; cl.bw[3][2] *= 3
    assert S.t_blk(cl, mo, T) <= base
    cl.c[3] *= 2
    assert S.t_blk(cl, mo, T) <= base
