"""GPU parity of the head redistribution (hexi_a2a_pack / hexi_a2a_unpack) against the CPU oracle:
byte-exact, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import a2a
from paper_2605_07569_amd import hexi

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bits(t):
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32).cpu().numpy()


def _case(s, n, d, dtype, head_lists, seed, extra_stride=0):
    print(f"\\n[a2a] s={s} heads={n} d={d} {dtype} ranks={len(head_lists)} listed={sum(len(h) for h in head_lists)} pad={extra_stride}", flush=True)
    g = torch.Generator().manual_seed(seed)
    wide = torch.randn((s, n * d + extra_stride), generator=g, dtype=torch.float32).to(dtype)
    x_cpu = wide[:, :n * d].reshape(s, n, d)
    wide_dev = wide.to(DEV)
    x = wide_dev[:, :n * d].view(s, n, d) if extra_stride == 0 else torch.as_strided(wide_dev, (s, n, d), (n * d + extra_stride, d, 1))
    total = sum(len(h) for h in head_lists) * s * d
    packed = torch.full((max(total, 1),), 7.0, dtype=dtype, device=DEV)
    hexi.hexi_a2a_pack(x, packed, head_lists)
    torch.cuda.synchronize()
    want = a2a.a2a_pack(_bits(x_cpu), head_lists)
    assert np.array_equal(_bits(packed)[:total], want)
    # unpack only where no head is listed twice
    flat = [h for heads in head_lists for h in heads]
    if len(set(flat)) == len(flat):
        y_wide = torch.full_like(wide_dev, 3.0)
        y = torch.as_strided(y_wide, (s, n, d), (n * d + extra_stride, d, 1))
        hexi.hexi_a2a_unpack(packed, y, head_lists)
        torch.cuda.synchronize()
        y0 = np.ascontiguousarray(_bits(torch.full((s, n, d), 3.0, dtype=dtype)))
        want_y = a2a.a2a_unpack(want, s, n, d, head_lists, y=y0)
        got = _bits(y_wide)[:, :n * d].reshape(s, n, d)
        assert np.array_equal(got, want_y)
        if extra_stride:   # the padding between tokens is not touched
            assert np.array_equal(_bits(y_wide)[:, n * d:], _bits(torch.full((s, extra_stride), 3.0, dtype=dtype)))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("d", [64, 128])
def test_pack_unpack_small_shapes(dtype, d):
    # uneven head counts per rank, non-adjacent heads, a rank with no head, heads that go nowhere,
    # token counts around the block size (32) and a single token
    for s in (1, 31, 32, 33, 777):
        _case(s, 12, d, dtype, [[11, 0, 5], [], [3], [8, 9, 1, 2, 6]], seed=s)
    _case(100, 8, d, dtype, [list(range(8))], seed=1)                      # identity
    _case(100, 8, d, dtype, [[7, 6, 5, 4, 3, 2, 1, 0]], seed=2)           # one rank, reversed (a sub-ring slice)
    _case(65, 5, d, dtype, [[0], [0, 1], [1, 4, 4]], seed=3)              # replicated heads: pack only
    _case(50, 6, d, dtype, [[4, 1], [0, 5, 2, 3]], seed=4, extra_stride=40)   # x is a slice of a wider buffer


def test_fused_qkv_shard_with_uneven_head_counts():
    # a pre-A2A shard of a 32/8-head GQA layer, Q, K and V fused along the head axis (48 heads), sent to
    # 3 ranks that own 16, 10 and 6 q heads and the kv heads their groups need (kv heads 2 and 3 replicated)
    nq, nkv, d, s = 32, 8, 128, 2048
    q_of = [list(range(0, 16)), list(range(16, 26)), list(range(26, 32))]
    lists = []
    for heads in q_of:
        kv = sorted({h // 4 for h in heads})
        lists.append(heads + [nq + k for k in kv] + [nq + nkv + k for k in kv])
    _case(s, nq + 2 * nkv, d, torch.bfloat16, lists, seed=9)


def test_full_size_shard_sampled():
    # configuration-4-sized shard: 32768 tokens x 48 fused heads x 128 (403 MB); every byte compared
    s, n, d = 32768, 48, 128
    lists = [list(range(0, 20)) + [32, 33, 40, 41], list(range(20, 32)) + [34, 35, 36, 37, 38, 39, 42, 43, 44, 45, 46, 47]]
    _case(s, n, d, torch.bfloat16, lists, seed=11)
