"""Pins of the head-redistribution oracle (oracle/a2a.py): the definition by loops, a hand-written
example, sizes from the paper's volume formula, and the inverse property."""
import numpy as np

from oracle import a2a


def test_hand_example():
    # 2 tokens, 3 heads, d = 2; element value 100*t + 10*h + c.  Rank 0 gets head 2, rank 1 heads 0 and 1.
    x = np.array([[[100 * t + 10 * h + c for c in range(2)] for h in range(3)] for t in range(2)], dtype=np.int32)
    want = [20, 21, 120, 121,                      # rank 0: tokens 0, 1 of head 2
            0, 1, 10, 11, 100, 101, 110, 111]      # rank 1: token 0 (heads 0, 1), token 1 (heads 0, 1)
    assert a2a.a2a_pack(x, [[2], [0, 1]]).tolist() == want
    assert a2a.a2a_pack_loops(x, [[2], [0, 1]]).tolist() == want


def test_vectorised_form_equals_definition():
    rng = np.random.default_rng(3)
    for s, n, d, lists in ((5, 7, 4, [[6, 0, 3], [1], [5, 2, 4]]), (1, 4, 8, [[3, 3, 0]]), (3, 2, 2, [[], [1, 0]])):
        x = rng.integers(-1000, 1000, size=(s, n, d)).astype(np.int64)
        assert np.array_equal(a2a.a2a_pack(x, lists), a2a.a2a_pack_loops(x, lists))


def test_part_sizes_follow_the_volume_formula():
    # App. A.4: the volume from a device to rank j is s * n_j * d elements per tensor
    s, d, lists = 11, 16, [[0, 5, 2], [1], [3, 4, 6, 7]]
    offs, total = a2a.part_offsets(s, d, lists)
    assert offs == [0, s * 3 * d, s * 4 * d] and total == s * 8 * d
    x = np.arange(s * 8 * d, dtype=np.int64).reshape(s, 8, d)
    buf = a2a.a2a_pack(x, lists)
    assert buf.size == total
    for j, heads in enumerate(lists):
        part = buf[offs[j]:offs[j] + s * len(heads) * d].reshape(s, len(heads), d)
        assert np.array_equal(part, x[:, heads, :])


def test_unpack_inverts_pack_and_keeps_unnamed_heads():
    rng = np.random.default_rng(4)
    s, n, d = 9, 6, 8
    x = rng.standard_normal((s, n, d)).astype(np.float32)
    lists = [[4, 1], [0, 5, 2, 3]]                     # a partition of the heads
    assert np.array_equal(a2a.a2a_unpack(a2a.a2a_pack(x, lists), s, n, d, lists), x)
    lists = [[4], [0, 2]]                              # heads 1, 3, 5 go nowhere
    y = np.full((s, n, d), 7.0, dtype=np.float32)
    y = a2a.a2a_unpack(a2a.a2a_pack(x, lists), s, n, d, lists, y=y)
    for h in range(n):
        assert np.array_equal(y[:, h, :], x[:, h, :] if h in (4, 0, 2) else np.full((s, d), 7.0, dtype=np.float32))
    # identity list: the send buffer is x itself
    assert np.array_equal(a2a.a2a_pack(x, [list(range(n))]), x.reshape(-1))
