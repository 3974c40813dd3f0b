"""Exhaustive search over HexiSeq's schedule space for tiny clusters (Sec. 4.1: the space the hierarchical
scheduler of Sec. 4.3 samples).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only ``tests/`` may import this module.  It enumerates EVERY valid
schedule -- every partition of the devices into A2A groups (ring order by smallest device, the scheduler's
convention), every split of L_tot between the groups in multiples of the token quantum, every split of a
group's length between its devices (a device may hold no tokens) and every split of the N heads between a
group's devices (a device may hold no heads) -- prices each with the performance model of oracle.scheduler
(App. A) and returns the cheapest one that passes the memory filter.  Nothing here is shared with the
scheduler's own search code or with the library; it exists so that the search has something to be measured
against that does not depend on the search.
"""
from . import scheduler as S


def set_partitions(items):
    """All partitions of a list into non-empty blocks; blocks ordered by their smallest element."""
    if not items:
        yield []
        return
    first, rest = items[0], items[1:]
    for part in set_partitions(rest):
        # `first` is smaller than everything in `rest`: it opens a new leading block or joins an existing one
        yield [[first]] + part
        for i in range(len(part)):
            yield [[first] + part[i]] + part[:i] + part[i + 1:]


def compositions(total, parts, minimum):
    """All tuples of `parts` integers >= minimum that sum to `total`."""
    if parts == 1:
        if total >= minimum:
            yield (total,)
        return
    for x in range(minimum, total - minimum * (parts - 1) + 1):
        for tail in compositions(total - x, parts - 1, minimum):
            yield (x,) + tail


def product_of(lists):
    if not lists:
        yield ()
        return
    for head in lists[0]:
        for tail in product_of(lists[1:]):
            yield (head,) + tail


def all_schedules(cl, mo, q):
    units = mo.l_tot // q
    assert units * q == mo.l_tot
    for groups in set_partitions(list(range(cl.n))):
        groups = sorted((sorted(g) for g in groups), key=lambda g: g[0])
        K = len(groups)
        for lens_u in compositions(units, K, 1):
            per_group = []
            for g, lu in zip(groups, lens_u):
                per_group.append([(s, h) for s in compositions(lu, len(g), 0) for h in compositions(mo.N, len(g), 0)])
            for choice in product_of(per_group):
                s_pre, n_heads = [0] * cl.n, [0] * cl.n
                for g, (s, h) in zip(groups, choice):
                    for d, sv, hv in zip(g, s, h):
                        s_pre[d], n_heads[d] = sv * q, hv
                yield S.Schedule(groups, [u * q for u in lens_u], s_pre, n_heads)


def optimum(cl, mo, q):
    """(best schedule, its T_blk, number of valid schedules, number that pass the memory filter)."""
    best, best_c, n_all, n_ok = None, S.INF, 0, 0
    for T in all_schedules(cl, mo, q):
        n_all += 1
        if not S.feasible(cl, mo, T):
            continue
        n_ok += 1
        c = S.t_blk(cl, mo, T)
        if c < best_c:
            best, best_c = T, c
    return best, best_c, n_all, n_ok
