"""CPU oracle of HexiSeq's analytical performance model and hierarchical scheduler.

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only ``tests/`` may import this module.  It shares no code
with the library's C++ scheduler.  Plain Python floats (IEEE doubles) and ints, every formula in the
paper's notation and order.

Cost model (Sec. 4.2, App. A): per device d with profile (c_d, b_d, m_d), group G(d) = G_k of
sequence length L_k, pre-A2A shard s_d and head count n_d:
    T_nonattn(d) = max(72 B s_d H^2 / c_d, 40 B s_d H P / b_d)                               (App. A.3)
    V(d->j)      = 3 B s_d (n_j d_h) P,   T_A2A(G_k) = 4 max_{d != j in G_k}(alpha_dj + beta_dj V(d->j))   (App. A.4)
    Msg(d,t)     = 4 B L_src(t) (n_d d_h) P,   F_step(d,t) = 16 B L_G(d) L_src(t) (n_d d_h)
    T_step(t)    = max_d F_step/c_d (t = 0),  max_d max(F_step/c_d, comm(d,t)) (t > 0)         (App. A.4, Eq. 12)
    T_blk        = max_d T_nonattn + max_k T_A2A + sum_t T_step(t)                             (Sec. 4.2)
    Mem_act(d)   = B P (gamma s_d H + 2 L_G(d) n_d d_h) <= m_d - M_static_d                    (App. A.2)

Readings where the paper is silent or at odds with itself:
 r1  Every A2A group holds all heads: sum_{d in G_k} n_d = N_heads for every k (the text's "globally"
     cannot hold once there is more than one group, since each group attends with all heads over its block).
 r2  Groups form a ring in the order of their smallest device index; at step t group k receives the KV
     block that originated in group (k - t) mod K, always from its ring predecessor (k - 1) mod K.
 r3  Heads are laid out over a group's devices in device order (device i holds a contiguous range of n_i
     heads).  The senders of device d are the predecessor group's devices whose ranges overlap d's; each sends
     its overlap and they transfer in parallel: comm(d,t) = max_u(alpha_ud + beta_ud Msg(d,t) overlap(u,d)/n_d).
     With identical layouts this is the paper's single-peer formula.  A device with n_d = 0 has no ring traffic.
 r4  Stage I: edge weight = min of the two directions' bandwidth; agglomeration levels = connected components
     of the edges at or above each distinct bandwidth, walked from the fastest down and stopped before the
     first level whose bandwidth is more than `gap_ratio` times slower than the previous one; the three
     baseline layouts (singletons = Ring, one group = Ulysses, equal consecutive groups of every divisor
     size = USP meshes) are always candidates; ranking by the smallest intra-group edge bandwidth (a group
     of one counts as infinitely fast), ties by fewer groups, then by first appearance.
 r4b Stage I super-node abstraction (Alg. 1 line 2): a group G_k of a retained partition is summarised by
     C_k = sum c_d, Bw_k = sum b_d, its memory proxy min_d (m_d - M_static_d) (the activation budget of its tightest
     device), its size, the mean startup latency and mean inverse bandwidth over its ordered intra-group device pairs
     (both 0 for a group of one), and the same two means over the edges u -> d from its ring predecessor's devices to
     its own (the inter-group edges that carry its ring traffic).  Stage II sees only these summaries: a group-level
     plan (L_1..L_K) is priced as if every group were one device that splits its tokens and heads evenly,
         T_nonattn = max_k max(72 B L_k H^2 / C_k, 40 B L_k H P / Bw_k),
         T_A2A     = max_k 4 (alpha_k + beta_k 3 B (L_k / |G_k|) ((N / |G_k|) d_h) P)       (0 for |G_k| = 1),
         T_step(t) = max_k max(16 B L_k L_src(t) (N d_h) / C_k,  [t > 0] alpha'_k + beta'_k 4 B L_src(t) ((N / |G_k|) d_h) P),
     and kept only if B P (gamma (L_k / |G_k|) H + 2 L_k (N / |G_k|) d_h) fits every group's memory proxy.  On a
     cluster of identical devices with identical links this equals the full model of the even schedule.
 r5  Stage II seeds: uniform (L_k proportional to the group's device count: the symmetric baselines),
     compute-proportional, square-root-compute, memory-capped (compute-proportional, groups clipped to the
     L their memory proxy admits under an even split of tokens and heads, the excess going to the others in
     proportion to compute; a group's cap is the largest multiple of q not above budget / bytes-per-token, i.e.
     floor(x / q) q evaluated in floating point); perturbations: `perturb` = 1/32 of L_tot moved between
     ring-adjacent groups, both directions.  Lengths are multiples of the token quantum q (largest-remainder
     rounding).  Scored on the super-node summaries (r4b); the best M2 of each partition go on, and a plan whose
     initial rank-level assignment (r6) fails the per-device memory filter is dropped there.
 r6  Stage III initial assignment: s_d and n_d proportional to c_d within the group (uniform for the
     uniform seed), largest-remainder rounding, ties to the lower device index.  Candidate pairs: ordered
     pairs of distinct devices in the same or ring-adjacent groups, lexicographic.  Moves per pair, in this
     order: `move_tokens` tokens from d_a to d_b (the group lengths follow when the groups differ), then one
     head from d_a to d_b (same group only).  First strictly improving feasible move is taken.
"""
import math

INF = float("inf")


class Cluster:
    def __init__(self, c, b, m, m_static, alpha, bw):
        self.n = len(c)
        self.c, self.b, self.m, self.m_static = list(c), list(b), list(m), list(m_static)
        self.alpha = [list(r) for r in alpha]      # alpha[i][j]: startup latency i -> j (s)
        self.bw = [list(r) for r in bw]            # bw[i][j]: bandwidth i -> j (bytes/s); beta = 1 / bw


class Model:
    def __init__(self, l_tot, batch, hidden, head_dim, n_heads, dtype_bytes, gamma_act=2.0):
        self.l_tot, self.B, self.H, self.d_h, self.N, self.P, self.gamma = l_tot, batch, hidden, head_dim, n_heads, dtype_bytes, gamma_act


class Schedule:
    def __init__(self, groups, l_group, s_pre, n_heads):
        self.groups = [list(g) for g in groups]    # ring order; devices ascending inside
        self.l_group = list(l_group)               # L_k
        self.s_pre = list(s_pre)                   # per device
        self.n_heads = list(n_heads)               # per device

    def copy(self):
        return Schedule(self.groups, self.l_group, self.s_pre, self.n_heads)

    def key(self):
        return (tuple(tuple(g) for g in self.groups), tuple(self.l_group), tuple(self.s_pre), tuple(self.n_heads))


# ------------------------------------------------------------------ cost model

def t_nonattn(cl, mo, T, d):
    flops = 72.0 * mo.B * T.s_pre[d] * mo.H * mo.H
    vol = 40.0 * mo.B * T.s_pre[d] * mo.H * mo.P
    return max(flops / cl.c[d], vol / cl.b[d])


def t_a2a(cl, mo, T, k):
    worst = 0.0
    g = T.groups[k]
    for d in g:
        for j in g:
            if j == d:
                continue
            vol = 3.0 * mo.B * T.s_pre[d] * (T.n_heads[j] * mo.d_h) * mo.P
            worst = max(worst, cl.alpha[d][j] + vol / cl.bw[d][j])
    return 4.0 * worst


def head_ranges(T, k):
    lo, out = 0, {}
    for d in T.groups[k]:
        out[d] = (lo, lo + T.n_heads[d])
        lo += T.n_heads[d]
    return out


def t_step(cl, mo, T, t):
    K = len(T.groups)
    worst = 0.0
    for k in range(K):
        src = (k - t) % K
        pred = (k - 1) % K
        mine = head_ranges(T, k)
        theirs = head_ranges(T, pred)
        for d in T.groups[k]:
            flops = 16.0 * mo.B * T.l_group[k] * T.l_group[src] * (T.n_heads[d] * mo.d_h)
            cost = flops / cl.c[d]
            if t > 0 and T.n_heads[d] > 0:
                msg = 4.0 * mo.B * T.l_group[src] * (T.n_heads[d] * mo.d_h) * mo.P
                comm = 0.0
                for u in T.groups[pred]:
                    ov = min(mine[d][1], theirs[u][1]) - max(mine[d][0], theirs[u][0])
                    if ov > 0:
                        comm = max(comm, cl.alpha[u][d] + (msg * ov / T.n_heads[d]) / cl.bw[u][d])
                cost = max(cost, comm)
            worst = max(worst, cost)
    return worst


def t_blk(cl, mo, T):
    a = max(t_nonattn(cl, mo, T, d) for d in range(cl.n))
    b = max(t_a2a(cl, mo, T, k) for k in range(len(T.groups)))
    c = 0.0
    for t in range(len(T.groups)):
        c += t_step(cl, mo, T, t)
    return a + b + c


def mem_act(cl, mo, T, d, k):
    return mo.B * mo.P * (mo.gamma * T.s_pre[d] * mo.H + 2.0 * T.l_group[k] * (T.n_heads[d] * mo.d_h))


def feasible(cl, mo, T):
    for k, g in enumerate(T.groups):
        for d in g:
            if cl.m_static[d] + mem_act(cl, mo, T, d, k) > cl.m[d]:
                return False
    return True


def valid(cl, mo, T):
    """Structural constraints of a schedule (Sec. 4.1 with reading r1)."""
    seen = sorted(d for g in T.groups for d in g)
    if seen != list(range(cl.n)) or sum(T.l_group) != mo.l_tot:
        return False
    for k, g in enumerate(T.groups):
        if sum(T.s_pre[d] for d in g) != T.l_group[k] or sum(T.n_heads[d] for d in g) != mo.N:
            return False
        if any(T.s_pre[d] < 0 or T.n_heads[d] < 0 for d in g) or T.l_group[k] <= 0:
            return False
    return True


# ------------------------------------------------------------------ scheduler

def largest_remainder(total, weights, quantum=1):
    """Integers that are multiples of `quantum`, sum to `total`, proportional to `weights`; leftover units go
    to the largest fractional parts, ties to the lower index."""
    units = total // quantum
    wsum = 0.0
    for w in weights:
        wsum += w
    exact = [units * (w / wsum) for w in weights]
    base = [int(math.floor(e)) for e in exact]
    left = units - sum(base)
    order = sorted(range(len(weights)), key=lambda i: (-(exact[i] - base[i]), i))
    for i in order[:left]:
        base[i] += 1
    return [x * quantum for x in base]


def components(n, bw, threshold):
    parent = list(range(n))

    def find(x):
        while parent[x] != x:
            parent[x] = parent[parent[x]]
            x = parent[x]
        return x
    for i in range(n):
        for j in range(i + 1, n):
            if min(bw[i][j], bw[j][i]) >= threshold:
                ri, rj = find(i), find(j)
                if ri != rj:
                    parent[max(ri, rj)] = min(ri, rj)
    groups = {}
    for d in range(n):
        groups.setdefault(find(d), []).append(d)
    return [groups[r] for r in sorted(groups)]


def intra_bandwidth(groups, bw):
    worst = INF
    for g in groups:
        for i in g:
            for j in g:
                if i != j:
                    worst = min(worst, min(bw[i][j], bw[j][i]))
    return worst


def partition_topology(cl, m1=64, gap_ratio=4.0):
    cands = []

    def add(groups):
        key = tuple(tuple(g) for g in groups)
        if key not in [c[0] for c in cands]:
            cands.append((key, len(cands)))
    n = cl.n
    add([[d] for d in range(n)])                       # Ring baseline
    add([list(range(n))])                              # Ulysses baseline
    for size in range(2, n):                           # USP meshes
        if n % size == 0:
            add([list(range(a, a + size)) for a in range(0, n, size)])
    levels = sorted({min(cl.bw[i][j], cl.bw[j][i]) for i in range(n) for j in range(i + 1, n)}, reverse=True)
    prev = None
    for lv in levels:
        if prev is not None and prev > gap_ratio * lv:
            break
        add(components(n, cl.bw, lv))
        prev = lv
    n_base = 2 + sum(1 for size in range(2, n) if n % size == 0)
    ranked = sorted(cands, key=lambda c: (-intra_bandwidth(c[0], cl.bw), len(c[0]), c[1]))
    keep = [c for c in ranked if c[1] < n_base]        # the baselines always stay
    for c in ranked:
        if len(keep) >= max(m1, n_base):
            break
        if c[1] >= n_base:
            keep.append(c)
    keep.sort(key=lambda c: (-intra_bandwidth(c[0], cl.bw), len(c[0]), c[1]))
    return [[list(g) for g in c[0]] for c in keep]


class SuperNode:
    """Stage I summary of one A2A group (reading r4b)."""
    def __init__(self, size, compute, mem_bw, mem, alpha_in, beta_in, alpha_ring, beta_ring):
        self.size, self.compute, self.mem_bw, self.mem = size, compute, mem_bw, mem
        self.alpha_in, self.beta_in = alpha_in, beta_in            # mean over ordered intra-group pairs
        self.alpha_ring, self.beta_ring = alpha_ring, beta_ring    # mean over edges predecessor group -> this group


def abstract_super_nodes(cl, groups):
    K = len(groups)
    nodes = []
    for k, g in enumerate(groups):
        a_in = b_in = 0.0
        pairs = 0
        for d in g:
            for j in g:
                if d != j:
                    a_in += cl.alpha[d][j]
                    b_in += 1.0 / cl.bw[d][j]
                    pairs += 1
        if pairs:
            a_in, b_in = a_in / pairs, b_in / pairs
        a_r = b_r = 0.0
        if K > 1:
            pred = groups[(k - 1) % K]
            for u in pred:
                for d in g:
                    a_r += cl.alpha[u][d]
                    b_r += 1.0 / cl.bw[u][d]
            a_r, b_r = a_r / (len(pred) * len(g)), b_r / (len(pred) * len(g))
        nodes.append(SuperNode(len(g), sum(cl.c[d] for d in g), sum(cl.b[d] for d in g),
                               min(cl.m[d] - cl.m_static[d] for d in g), a_in, b_in, a_r, b_r))
    return nodes


def supernode_cost(nodes, mo, lens):
    """Coarse T_blk of a group-level plan: every group one device, tokens and heads split evenly inside it."""
    K = len(nodes)
    nonattn = max(max(72.0 * mo.B * lens[k] * mo.H * mo.H / nodes[k].compute, 40.0 * mo.B * lens[k] * mo.H * mo.P / nodes[k].mem_bw)
                  for k in range(K))
    a2a = 0.0
    for k, sn in enumerate(nodes):
        if sn.size > 1:
            vol = 3.0 * mo.B * (lens[k] / sn.size) * ((mo.N / sn.size) * mo.d_h) * mo.P
            a2a = max(a2a, 4.0 * (sn.alpha_in + sn.beta_in * vol))
    ring = 0.0
    for t in range(K):
        worst = 0.0
        for k, sn in enumerate(nodes):
            src = (k - t) % K
            cost = 16.0 * mo.B * lens[k] * lens[src] * (mo.N * mo.d_h) / sn.compute
            if t > 0:
                msg = 4.0 * mo.B * lens[src] * ((mo.N / sn.size) * mo.d_h) * mo.P
                cost = max(cost, sn.alpha_ring + sn.beta_ring * msg)
            worst = max(worst, cost)
        ring += worst
    return nonattn + a2a + ring


def supernode_feasible(nodes, mo, lens):
    for k, sn in enumerate(nodes):
        if mo.B * mo.P * (mo.gamma * (lens[k] / sn.size) * mo.H + 2.0 * lens[k] * ((mo.N / sn.size) * mo.d_h)) > sn.mem:
            return False
    return True


def initialize_assignment(cl, mo, groups, l_group, uniform, q):
    s_pre, n_heads = [0] * cl.n, [0] * cl.n
    for k, g in enumerate(groups):
        w = [1.0 if uniform else cl.c[d] for d in g]
        for d, v in zip(g, largest_remainder(l_group[k], w, q)):
            s_pre[d] = v
        for d, v in zip(g, largest_remainder(mo.N, w, 1)):
            n_heads[d] = v
    return Schedule(groups, l_group, s_pre, n_heads)


def generate_candidates(cl, mo, groups, q, perturb):
    """Group-level plans of one partition, from the groups' aggregate compute and memory proxy (the super-node
    summaries) alone: [(lens, uniform_flag), ...] in a fixed order."""
    K = len(groups)
    comp = [sum(cl.c[d] for d in g) for g in groups]
    seeds = []
    seeds.append((largest_remainder(mo.l_tot, [float(len(g)) for g in groups], q), True))
    seeds.append((largest_remainder(mo.l_tot, comp, q), False))
    seeds.append((largest_remainder(mo.l_tot, [math.sqrt(x) for x in comp], q), False))
    # memory-capped: per group the largest L its tightest device admits under an even split of tokens and heads
    cap = []
    for g in groups:
        budget = min(cl.m[d] - cl.m_static[d] for d in g)
        per_token = mo.B * mo.P * (mo.gamma * mo.H / len(g) + 2.0 * (mo.N / len(g)) * mo.d_h)
        cap.append(int(math.floor(max(0.0, budget / per_token) / q)) * q)
    lens = largest_remainder(mo.l_tot, comp, q)
    for _ in range(K):
        over = [k for k in range(K) if lens[k] > cap[k]]
        if not over:
            break
        excess = sum(lens[k] - cap[k] for k in over)
        for k in over:
            lens[k] = cap[k]
        free = [k for k in range(K) if lens[k] < cap[k]]
        if not free:
            break
        extra = largest_remainder(excess, [comp[k] for k in free], q)
        for k, e in zip(free, extra):
            lens[k] += e
    if sum(lens) == mo.l_tot:
        seeds.append((lens, False))
    out = []

    def add(lens, uniform):
        if all(x > 0 for x in lens) and (tuple(lens), uniform) not in [(tuple(a), b) for a, b in out]:
            out.append((list(lens), uniform))
    delta = (int(mo.l_tot * perturb) // q) * q
    for lens, uniform in seeds:
        add(lens, uniform)
    for lens, uniform in seeds:
        if K > 1 and delta > 0:
            for k in range(K):
                for nb in ((k + 1) % K, (k - 1) % K):
                    if nb != k and lens[k] > delta:
                        moved = list(lens)
                        moved[k] -= delta
                        moved[nb] += delta
                        add(moved, False)
    return out


def candidate_pairs(T):
    K = len(T.groups)
    group_of = {}
    for k, g in enumerate(T.groups):
        for d in g:
            group_of[d] = k
    pairs = []
    for a in sorted(group_of):
        for b in sorted(group_of):
            if a == b:
                continue
            ka, kb = group_of[a], group_of[b]
            if ka == kb or (kb - ka) % K == 1 or (ka - kb) % K == 1:
                pairs.append((a, b, ka, kb))
    return pairs


def propose_moves(T, a, b, ka, kb, move_tokens):
    moves = []
    if T.s_pre[a] >= move_tokens and (ka == kb or T.l_group[ka] > move_tokens):
        m = T.copy()
        m.s_pre[a] -= move_tokens
        m.s_pre[b] += move_tokens
        if ka != kb:
            m.l_group[ka] -= move_tokens
            m.l_group[kb] += move_tokens
        moves.append(m)
    if ka == kb and T.n_heads[a] >= 1:
        m = T.copy()
        m.n_heads[a] -= 1
        m.n_heads[b] += 1
        moves.append(m)
    return moves


def refine(cl, mo, T, i_max, move_tokens):
    C = t_blk(cl, mo, T)
    improved, i = True, 0
    while improved and i < i_max:
        improved, i = False, i + 1
        for a, b, ka, kb in candidate_pairs(T):
            done = False
            for m in propose_moves(T, a, b, ka, kb, move_tokens):
                if feasible(cl, mo, m):
                    c2 = t_blk(cl, mo, m)
                    if c2 < C:
                        T, C, improved, done = m, c2, True, True
                        break
            if done:
                break
    return T, C


def solve(cl, mo, m1=64, m2=16, i_max=100, gap_ratio=4.0, q=64, perturb=1.0 / 32, move_tokens=None):
    if move_tokens is None:
        move_tokens = max(1, mo.l_tot // (q * cl.n * 16)) * q
    best, best_c = None, INF
    for groups in partition_topology(cl, m1, gap_ratio):
        nodes = abstract_super_nodes(cl, groups)
        scored = []
        for idx, (lens, uniform) in enumerate(generate_candidates(cl, mo, groups, q, perturb)):
            if supernode_feasible(nodes, mo, lens):
                scored.append((supernode_cost(nodes, mo, lens), idx, lens, uniform))
        scored.sort(key=lambda x: (x[0], x[1]))
        for _, _, lens, uniform in scored[:m2]:
            T = initialize_assignment(cl, mo, groups, lens, uniform, q)
            if not feasible(cl, mo, T):
                continue
            T, C = refine(cl, mo, T, i_max, move_tokens)
            if C < best_c:
                best, best_c = T, C
    return best, best_c
