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


# ---------------------------------------------------------------------------------------------------------------
# Stage I-III pins written out by hand (Sec. 4.3; Alg. 1).  None of them re-runs the search to get its expectation.

def _toy_cluster(c, budgets=None, bw=1e30, alpha=0.0):
    """Devices with compute c[d], unlimited memory bandwidth, activation budget budgets[d] (m_static = 0) and
    identical links."""
    n = len(c)
    budgets = budgets or [1e18] * n
    return S.Cluster(list(c), [1e30] * n, list(budgets), [0.0] * n, [[0.0 if i == j else alpha for j in range(n)] for i in range(n)],
                     [[1e30 if i == j else bw for j in range(n)] for i in range(n)])


def test_memory_capped_seed_with_a_binding_cap_by_hand():
    """Stage II, memory-capped seed.  B = 1, P = 2, H = 1000, N = 4, d_h = 100, gamma = 2, L_tot = 4096, q = 64.
    A group of one device needs B P (gamma H + 2 N d_h) = 2 (2000 + 800) = 5600 bytes per token of L_k.
    Two groups of one device each, equal compute: the compute-proportional split is (2048, 2048).  Group 1 has an
    activation budget of 5.6e6 bytes = 1000 tokens -> cap = floor(1000 / 64) 64 = 960; it is clipped to 960 and the
    excess 1088 goes to group 0: (3136, 960).  Perturbations move L_tot / 32 = 128 tokens either way."""
    mo = S.Model(4096, 1, 1000, 100, 4, 2)
    cl = _toy_cluster([1e12, 1e12], budgets=[1e18, 5.6e6])
    got = S.generate_candidates(cl, mo, [[0], [1]], 64, 1.0 / 32)
    assert got == [([2048, 2048], True), ([2048, 2048], False), ([3136, 960], False),
                   ([1920, 2176], False), ([2176, 1920], False), ([3008, 1088], False), ([3264, 832], False)]
    # one token less of budget: 999 tokens -> still 15 quanta; one quantum boundary lower at 959 tokens
    cl = _toy_cluster([1e12, 1e12], budgets=[1e18, 5600.0 * 959])
    assert ([3200, 896], False) in S.generate_candidates(cl, mo, [[0], [1]], 64, 1.0 / 32)
    # three groups with compute 2 : 1 : 1 -> (2048, 1024, 1024); group 2 capped at floor(700 / 64) 64 = 640; its excess
    # of 384 = 6 quanta goes to groups 0 and 1 in proportion to compute (4 and 2 quanta): (2304, 1152, 640)
    cl = _toy_cluster([2e12, 1e12, 1e12], budgets=[1e18, 1e18, 5600.0 * 700])
    got = S.generate_candidates(cl, mo, [[0], [1], [2]], 64, 1.0 / 32)
    assert got[:2] == [([1408, 1344, 1344], True), ([2048, 1024, 1024], False)]      # uniform: 22 + 21 + 21 quanta
    assert ([2304, 1152, 640], False) in got
    # a cap that nothing can absorb (every group capped below its share): no memory-capped seed, the others stay
    cl = _toy_cluster([1e12, 1e12], budgets=[5600.0 * 1000, 5600.0 * 1000])
    assert S.generate_candidates(cl, mo, [[0], [1]], 64, 1.0 / 32)[:2] == [([2048, 2048], True), ([2048, 2048], False)]


def test_perturbation_set_by_hand():
    """Stage II candidates of two groups of one device with compute 3 : 1, L_tot = 4096, q = 64 (64 quanta), no
    memory pressure.  Seeds: uniform (32, 32 quanta); compute-proportional (48, 16); square-root-compute: weights
    sqrt(3) : 1 = 0.63397 : 0.36603 -> 40.57, 23.43 quanta -> 40 + 23 and the spare quantum to the larger fraction:
    (41, 23) = (2624, 1472); the memory-capped seed equals the compute-proportional one.  Each seed is followed, in
    seed order, by itself with 128 tokens moved from group 0 to its neighbour and from group 1 to its neighbour."""
    mo = S.Model(4096, 1, 1000, 100, 4, 2)
    cl = _toy_cluster([3e12, 1e12])
    assert S.generate_candidates(cl, mo, [[0], [1]], 64, 1.0 / 32) == [
        ([2048, 2048], True), ([3072, 1024], False), ([2624, 1472], False),
        ([1920, 2176], False), ([2176, 1920], False),
        ([2944, 1152], False), ([3200, 896], False),
        ([2496, 1600], False), ([2752, 1344], False)]
    # three equal groups, 192 tokens, q = 64, perturb 1/3 -> delta 64: from (64, 64, 64) nothing can move (a group must
    # keep more than delta); from 384 tokens (128 each) every group gives 64 to its ring successor, then to its predecessor
    cl3 = _toy_cluster([1e12, 1e12, 1e12])
    assert S.generate_candidates(cl3, S.Model(192, 1, 1000, 100, 4, 2), [[0], [1], [2]], 64, 1.0 / 3) == [([64, 64, 64], True), ([64, 64, 64], False)]
    got = S.generate_candidates(cl3, S.Model(384, 1, 1000, 100, 4, 2), [[0], [1], [2]], 64, 1.0 / 6)
    assert got == [([128, 128, 128], True), ([128, 128, 128], False),
                   ([64, 192, 128], False), ([64, 128, 192], False),        # group 0 gives to group 1, then to group 2
                   ([128, 64, 192], False), ([192, 64, 128], False),        # group 1 gives to group 2, then to group 0
                   ([192, 128, 64], False), ([128, 192, 64], False)]        # group 2 gives to group 0, then to group 1


def test_candidate_pairs_by_hand():
    """Stage III candidate pairs: ordered pairs of distinct devices in the same or ring-adjacent groups, lexicographic,
    each with its two group indices."""
    T = S.Schedule([[0, 1], [2]], [128, 64], [64, 64, 64], [2, 2, 4])
    assert S.candidate_pairs(T) == [(0, 1, 0, 0), (0, 2, 0, 1), (1, 0, 0, 0), (1, 2, 0, 1), (2, 0, 1, 0), (2, 1, 1, 0)]
    # a ring of four groups of one: the opposite groups (0, 2) and (1, 3) are not adjacent
    T = S.Schedule([[0], [1], [2], [3]], [64] * 4, [64] * 4, [4] * 4)
    assert [(a, b) for a, b, _, _ in S.candidate_pairs(T)] == [(0, 1), (0, 3), (1, 0), (1, 2), (2, 1), (2, 3), (3, 0), (3, 2)]
    # a ring of five with a group of two: device 1 (group 0) pairs with its own group and groups 1 and 4 only
    T = S.Schedule([[0, 1], [2], [3], [4], [5]], [64] * 5, [32, 32, 64, 64, 64, 64], [2, 2, 4, 4, 4, 4])
    assert [b for a, b, _, _ in S.candidate_pairs(T) if a == 1] == [0, 2, 5]


def test_proposed_moves_by_hand():
    """Per pair: first `move_tokens` tokens from a to b (group lengths follow between groups), then one head (same
    group only); a device cannot give what it does not hold, and a group never gives away its whole block."""
    T = S.Schedule([[0, 1], [2]], [128, 64], [64, 64, 64], [1, 3, 4])
    m = S.propose_moves(T, 0, 1, 0, 0, 64)
    assert [(x.l_group, x.s_pre, x.n_heads) for x in m] == [([128, 64], [0, 128, 64], [1, 3, 4]), ([128, 64], [64, 64, 64], [0, 4, 4])]
    m = S.propose_moves(T, 0, 2, 0, 1, 64)
    assert [(x.l_group, x.s_pre, x.n_heads) for x in m] == [([64, 128], [0, 64, 128], [1, 3, 4])]
    assert S.propose_moves(T, 2, 0, 1, 0, 64) == []                  # group 1 would be left without tokens
    T2 = S.Schedule([[0, 1]], [128], [0, 128], [0, 4])
    assert S.propose_moves(T2, 0, 1, 0, 0, 64) == []                 # nothing to give


def test_coordinate_descent_traced_by_hand():
    """Alg. 1 lines 9-19 on one group of two devices, c = (2e12, 1e12), free links, L_tot = 256, H = 1000, d_h = 100,
    N = 4, move budget 64 tokens, from s = (64, 192), n = (1, 3).
      T_nonattn(d) = 72 s_d 1e6 / c_d:  s = 64 -> 2.304e-3 (d0) / 4.608e-3 (d1); 128 -> 4.608e-3 / 9.216e-3;
                                         192 -> 6.912e-3 / 1.3824e-2; 256 -> 9.216e-3 / 1.8432e-2
      T_step = max_d 16 256^2 100 n_d / c_d = max(n_0 5.24288e-5, n_1 1.048576e-4)
      start: 1.3824e-2 + 3.145728e-4.
      pass 1: (0,1) tokens -> s = (0, 256) worse; (0,1) head -> n = (0, 4) worse; (1,0) tokens -> s = (128, 128):
              9.216e-3 + 3.145728e-4, accepted.
      pass 2: (0,1) both worse; (1,0) tokens -> s = (192, 64): 6.912e-3 + 3.145728e-4, accepted.
      pass 3: (0,1) both worse; (1,0) tokens -> (256, 0): 9.216e-3, worse; (1,0) head -> n = (2, 2): 6.912e-3 + 2.097152e-4, accepted.
      pass 4: (1,0) head -> n = (3, 1): 6.912e-3 + 1.572864e-4, accepted.
      pass 5: (0,1) tokens worse, head -> (2, 2) worse; (1,0) tokens worse, head -> (4, 0): 2.097152e-4, worse.  Stop."""
    cl, mo = _toy_cluster([2e12, 1e12]), S.Model(256, 1, 1000, 100, 4, 2)
    start = S.Schedule([[0, 1]], [256], [64, 192], [1, 3])
    assert S.t_blk(cl, mo, start) == pytest.approx(1.3824e-2 + 3.145728e-4, rel=1e-9)
    want = {1: ([128, 128], [1, 3], 9.216e-3 + 3.145728e-4), 2: ([192, 64], [1, 3], 6.912e-3 + 3.145728e-4),
            3: ([192, 64], [2, 2], 6.912e-3 + 2.097152e-4), 4: ([192, 64], [3, 1], 6.912e-3 + 1.572864e-4),
            5: ([192, 64], [3, 1], 6.912e-3 + 1.572864e-4), 100: ([192, 64], [3, 1], 6.912e-3 + 1.572864e-4)}
    for i_max, (s_pre, n_heads, cost) in want.items():
        T, C = S.refine(cl, mo, start.copy(), i_max, 64)
        assert (T.s_pre, T.n_heads) == (s_pre, n_heads), i_max
        assert C == pytest.approx(cost, rel=1e-9) and C == S.t_blk(cl, mo, T)
    # The same descent with a memory filter that binds (App. A.2): Mem_act(d0) = 2 (2000 s_0 + 51200 n_0) bytes:
    # s_0 = 192 needs at least 870400, s_0 = 128 needs 614400 + 102400 (n_0 - 1).  With 850000 bytes on device 0 the
    # token move of pass 2 is rejected although it is cheaper, and the descent goes on with heads:
    #   pass 2: (1,0) head -> n = (2, 2): 9.216e-3 + 2.097152e-4; pass 3: n = (3, 1): 9.216e-3 + 1.572864e-4;
    #   pass 4: n = (4, 0) needs 921600 bytes (and is worse): stop.
    cl = _toy_cluster([2e12, 1e12], budgets=[850000.0, 1e18])
    T, C = S.refine(cl, mo, start.copy(), 100, 64)
    assert (T.s_pre, T.n_heads) == ([128, 128], [3, 1]) and C == pytest.approx(9.216e-3 + 1.572864e-4, rel=1e-9)
    T, C = S.refine(cl, mo, start.copy(), 2, 64)
    assert (T.s_pre, T.n_heads) == ([128, 128], [2, 2]) and C == pytest.approx(9.216e-3 + 2.097152e-4, rel=1e-9)
    # an empty descent is not enough: the refined cost is strictly below the starting cost here
    assert C < S.t_blk(cl, mo, start)


def test_partition_ranking_and_truncation_by_hand():
    """Stage I on three nodes of two devices with intra-node links of 450, 300 and 200 GB/s and a 25 GB/s fabric.
    Baselines (always kept): Ring {0}..{5} (no intra-group edge: infinitely fast), Ulysses (slowest intra edge
    25 GB/s, 1 group), pairs {0,1}{2,3}{4,5} (200 GB/s, 3 groups), triples {0,1,2}{3,4,5} (25 GB/s, 2 groups).
    Agglomeration: at 450 GB/s {0,1} + four singletons (450 GB/s, 5 groups); at 300 GB/s {0,1}{2,3}{4}{5} (300 GB/s,
    4 groups); at 200 GB/s the pairs again; the next level, 25 GB/s, is 8x slower: stop.
    Ranking by slowest intra-group edge, then fewer groups."""
    arr = cluster_arrays([("h100", 2), ("a100", 2), ("a800", 2)])
    cl = _cluster(**arr)
    ring = [[d] for d in range(6)]
    a450, a300 = [[0, 1], [2], [3], [4], [5]], [[0, 1], [2, 3], [4], [5]]
    pairs, ulysses, triples = [[0, 1], [2, 3], [4, 5]], [list(range(6))], [[0, 1, 2], [3, 4, 5]]
    assert S.partition_topology(cl, m1=64) == [ring, a450, a300, pairs, ulysses, triples]
    assert S.partition_topology(cl, m1=5) == [ring, a450, pairs, ulysses, triples]      # the best non-baseline fills the fifth slot
    assert S.partition_topology(cl, m1=2) == [ring, pairs, ulysses, triples]            # the baselines always stay
    # a threshold of 1.2 stops the agglomeration after its first level (450 -> 300 GB/s is a 1.5x gap)
    assert S.partition_topology(cl, m1=64, gap_ratio=1.2) == [ring, a450, pairs, ulysses, triples]
    # direction-dependent links count with their slower direction
    slow = [list(r) for r in arr["bw"]]
    slow[1][0] = 100e9
    assert S.intra_bandwidth([[0, 1]], slow) == 100e9
    assert S.components(6, slow, 450e9) == [[0], [1], [2], [3], [4], [5]]


def test_super_node_summary_by_hand():
    """Alg. 1 line 2 on groups {0, 1} and {2}: c = (3, 1, 2)e12, b = (5, 7, 11)e11, activation budgets (9, 4, 6)e9;
    links 0<->1: 1e9 B/s one way and 2e9 the other, 1 ms / 3 ms startup; from group 0 to device 2: 4e9 and 1e9 B/s,
    2 ms and 4 ms; from device 2 to devices 0 and 1: 5e8 B/s, 6 ms and 10 ms."""
    bw = [[1e30, 1e9, 4e9], [2e9, 1e30, 1e9], [5e8, 5e8, 1e30]]
    al = [[0.0, 1e-3, 2e-3], [3e-3, 0.0, 4e-3], [6e-3, 10e-3, 0.0]]
    cl = S.Cluster([3e12, 1e12, 2e12], [5e11, 7e11, 11e11], [9e9 + 1e9, 4e9 + 1e9, 6e9 + 1e9], [1e9] * 3, al, bw)
    g0, g1 = S.abstract_super_nodes(cl, [[0, 1], [2]])
    assert (g0.size, g0.compute, g0.mem_bw, g0.mem) == (2, 4e12, 12e11, 4e9)
    assert (g1.size, g1.compute, g1.mem_bw, g1.mem) == (1, 2e12, 11e11, 6e9)
    assert g0.alpha_in == pytest.approx(2e-3) and g0.beta_in == pytest.approx((1e-9 + 0.5e-9) / 2)
    assert (g1.alpha_in, g1.beta_in) == (0.0, 0.0)
    assert g0.alpha_ring == pytest.approx(8e-3) and g0.beta_ring == pytest.approx(2e-9)              # edges 2 -> 0, 2 -> 1
    assert g1.alpha_ring == pytest.approx(3e-3) and g1.beta_ring == pytest.approx((0.25e-9 + 1e-9) / 2)   # edges 0 -> 2, 1 -> 2
    # coarse cost of the plan L = (3000, 1000) with B = 1, H = 1000, d_h = 100, N = 4, P = 2, by hand:
    #   T_nonattn: group 0: max(72 * 3000 * 1e6 / 4e12, 40 * 3000 * 1000 * 2 / 12e11) = max(0.054, 2e-4); group 1: 72e9 / 2e12 = 0.036
    #   T_A2A: group 0: V = 3 * 1500 * (2 * 100) * 2 = 1.8e6 B -> 4 (2e-3 + 0.75e-9 * 1.8e6) = 0.0134
    #   step 0: group 0: 16 * 3000^2 * 400 / 4e12 = 0.0144; group 1: 16 * 1000^2 * 400 / 2e12 = 0.0032
    #   step 1: compute 16 * 3000 * 1000 * 400 = 1.92e10 -> 0.0048 (group 0), 0.0096 (group 1);
    #           group 0 receives 4 * 1000 * (2 * 100) * 2 = 1.6e6 B: 8e-3 + 2e-9 * 1.6e6 = 0.0112;
    #           group 1 receives 4 * 3000 * (4 * 100) * 2 = 9.6e6 B: 3e-3 + 0.625e-9 * 9.6e6 = 0.009  -> max 0.0112
    mo = S.Model(4000, 1, 1000, 100, 4, 2)
    assert S.supernode_cost([g0, g1], mo, [3000, 1000]) == pytest.approx(0.054 + 0.0134 + 0.0144 + 0.0112, rel=1e-12)
    # memory proxy: group 0 needs 2 (2 * 1500 * 1000 + 2 * 3000 * 2 * 100) = 8.4e6 bytes, group 1 2 (2e6 + 8e5) = 5.6e6
    assert S.supernode_feasible([g0, g1], mo, [3000, 1000])
    g1.mem = 5.6e6 - 1.0
    assert not S.supernode_feasible([g0, g1], mo, [3000, 1000])


def test_super_node_cost_equals_the_full_model_on_symmetric_layouts():
    arr = cluster_arrays([("a100", 4)])
    cl, mo = _cluster(**arr), S.Model(**model_args(l_tot=32768))
    for groups in ([[0], [1], [2], [3]], [[0, 1, 2, 3]], [[0, 1], [2, 3]]):
        lens = [32768 // len(groups)] * len(groups)
        T = S.initialize_assignment(cl, mo, groups, lens, True, 64)
        assert S.supernode_cost(S.abstract_super_nodes(cl, groups), mo, lens) == pytest.approx(S.t_blk(cl, mo, T), rel=1e-12)
