"""Host logic of the C ABI, runnable without a GPU: the library loads, exports every symbol the header
declares, the integer bookkeeping is bit-exact against the brute-force oracle, and argument
validation returns the documented error codes before anything is launched."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

import oracle
from paper_2605_07569_amd import hexi
from paper_2605_07569_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    return set(re.findall(r"\b(hexi_[a-z0-9_]+)\s*\(", header))


def _dynamic_symbols(path):
    out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    return {line.split()[-1] for line in out.splitlines() if line.strip()}


def test_library_exports_every_declared_symbol():
    """Every function a header under include/ declares is exported by that header's library, the binding knows
    the same names, and nothing else leaves the libraries (no kernel stubs, no C++ library symbols)."""
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["hexi_attn.h", "hexi_probe.h"]
    declared = _declared("hexi_attn.h")
    assert {"hexi_shard_mask", "hexi_attn_fwd_chunk", "hexi_attn_merge_lse", "hexi_attn_bwd_chunk"} <= declared
    lib = hexi.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(hexi.EXPORTS)
    assert _dynamic_symbols(hexi.LIB_PATH) == declared
    assert "gfx950" in hexi.hexi_version()
    probe = hexi.load_probe()
    declared = _declared("hexi_probe.h")
    assert declared == set(hexi.PROBE_EXPORTS) and all(hasattr(probe, n) for n in declared)
    assert _dynamic_symbols(hexi.PROBE_LIB_PATH) == declared


def test_run_length_knob_round_trip():
    assert hexi.hexi_set_dkdv_run_len(3) == 0
    assert hexi.hexi_set_dkdv_run_len(-5) == 3      # negative values mean automatic
    assert hexi.hexi_set_dkdv_run_len(0) == 0


def _random_segs(rng, n_seg, max_len, max_gap):
    out, cur = [], int(rng.integers(0, max_gap + 1))
    for _ in range(n_seg):
        ln = int(rng.integers(1, max_len + 1))
        out.append((cur, ln))
        cur += ln + int(rng.integers(0, max_gap + 1))
    return out


def test_shard_mask_bit_exact_vs_bruteforce_random():
    rng = np.random.default_rng(123)
    for trial in range(40):
        qs = _random_segs(rng, int(rng.integers(1, 6)), 300, 200)
        ks = _random_segs(rng, int(rng.integers(1, 6)), 300, 200)
        tm, tn = [(128, 64), (64, 128), (7, 5), (1, 1), (1000, 777)][trial % 5]
        r = hexi.hexi_shard_mask(qs, ks, tm, tn)
        qp, kp = oracle.positions(qs), oracle.positions(ks)
        cls, n = oracle.mask_bruteforce(qp, kp, tm, tn)
        assert np.array_equal(r["q_pos"], qp.astype(np.int32))
        assert np.array_equal(r["kv_pos"], kp.astype(np.int32))
        assert r["n_pairs"] == n
        assert np.array_equal(r["tile_class"], cls)


def test_shard_mask_on_shrunken_configs_and_full_pair_counts():
    import json
    gold = json.load(open(os.path.join(ROOT, "tests", "golden", "config_pair_counts.json")))["n_pairs"]
    for idx in range(1, 6):
        w = wl.config(idx)
        total = sum(hexi.hexi_shard_mask(w.q_segs, ch, want_pos=False)["n_pairs"] for ch in w.chunks)
        assert total == gold[str(idx)]
    for idx, shrink in ((2, 64), (3, 128), (4, 128), (5, 256)):
        w = wl.config(idx, shrink=shrink)
        qp = oracle.positions(w.q_segs)
        for ch in w.chunks:
            r = hexi.hexi_shard_mask(w.q_segs, ch, 128, 64)
            cls, n = oracle.mask_bruteforce(qp, oracle.positions(ch), 128, 64)
            assert r["n_pairs"] == n and np.array_equal(r["tile_class"], cls)


def test_shard_mask_unaligned_and_degenerate():
    for qs, ks in (([(5, 1)], [(5, 1)]), ([(0, 1000)], [(0, 777)]), ([(3, 1)], [(4, 9)]), ([(100, 50)], [(0, 1)])):
        r = hexi.hexi_shard_mask(qs, ks, 128, 128)
        cls, n = oracle.mask_bruteforce(oracle.positions(qs), oracle.positions(ks), 128, 128)
        assert r["n_pairs"] == n and np.array_equal(r["tile_class"], cls)


def test_range_validation_errors():
    for bad in ([], [(0, 0)], [(-1, 4)], [(10, 5), (12, 3)], [(10, 5), (2, 3)], [(0, 1)] * 17):
        with pytest.raises(hexi.HexiError) as e:
            hexi.hexi_shard_mask(bad, [(0, 4)], 4, 4)
        assert e.value.code == hexi.HEXI_EINVAL
    with pytest.raises(hexi.HexiError) as e:
        hexi.hexi_shard_mask([(2 ** 31 - 4, 8)], [(0, 4)], 4, 4, want_pos=False, want_classes=False)
    assert e.value.code == hexi.HEXI_EUNSUPPORTED
    # adjacent segments are legal
    assert hexi.hexi_shard_mask([(0, 4), (4, 4)], [(0, 8)], 4, 4)["n_pairs"] == 36


def _call_fwd(desc, q_segs, kv_segs, ptrs, flags=0):
    lib = hexi.load()
    qr, k1 = hexi.make_range(q_segs)
    kr, k2 = hexi.make_range(kv_segs)
    vp = [ctypes.c_void_p(p) for p in ptrs]
    return lib.hexi_attn_fwd_chunk(ctypes.byref(desc), ctypes.byref(qr), ctypes.byref(kr), *vp, flags, None, 0, None)


def test_descriptor_validation_returns_codes_without_launching():
    good = (4096, 8192, 12288, 16384, 20480)  # fake 16-byte-aligned device addresses; never dereferenced on error
    d = hexi.make_desc(hexi.HEXI_BF16, 128, 8, 2, 0.088, (1024, 128), (256, 128))
    assert _call_fwd(d, [(0, 4)], [(0, 4)], (0,) + good[1:]) == hexi.HEXI_EINVAL          # null q
    assert _call_fwd(d, [(0, 4)], [(0, 4)], (4100,) + good[1:]) == hexi.HEXI_EALIGN       # misaligned q
    assert _call_fwd(d, [(0, 4)], [(0, 4)], good, flags=64) == hexi.HEXI_EINVAL           # unknown flag
    assert "flag" in hexi.hexi_last_error()
    bad = hexi.make_desc(hexi.HEXI_BF16, 96, 8, 2, 0.1, (768, 96), (192, 96))
    assert _call_fwd(bad, [(0, 4)], [(0, 4)], good) == hexi.HEXI_EUNSUPPORTED             # head_dim
    bad = hexi.make_desc(hexi.HEXI_BF16, 128, 8, 2, 0.1, ((1 << 22) + 8, 128), (256, 128))
    assert _call_fwd(bad, [(0, 4)], [(0, 4)], good) == hexi.HEXI_EUNSUPPORTED             # token stride beyond the 32-bit tile offsets
    bad = hexi.make_desc(7, 128, 8, 2, 0.1, (1024, 128), (256, 128))
    assert _call_fwd(bad, [(0, 4)], [(0, 4)], good) == hexi.HEXI_EUNSUPPORTED             # dtype
    bad = hexi.make_desc(hexi.HEXI_BF16, 128, 8, 3, 0.1, (1024, 128), (384, 128))
    assert _call_fwd(bad, [(0, 4)], [(0, 4)], good) == hexi.HEXI_EINVAL                   # 8 % 3 with NULL map
    bad = hexi.make_desc(hexi.HEXI_BF16, 128, 2, 2, 0.1, (256, 128), (256, 128), kv_of_q=[0, 2])
    assert _call_fwd(bad, [(0, 4)], [(0, 4)], good) == hexi.HEXI_EINVAL                   # map out of range
    bad = hexi.make_desc(hexi.HEXI_BF16, 128, 8, 2, 0.1, (1020, 128), (256, 128))
    assert _call_fwd(bad, [(0, 4)], [(0, 4)], good) == hexi.HEXI_EALIGN                   # stride not 16 B
    bad = hexi.make_desc(hexi.HEXI_BF16, 128, 8, 2, 0.1, (1024, 64), (256, 128))
    assert _call_fwd(bad, [(0, 4)], [(0, 4)], good) == hexi.HEXI_EINVAL                   # head stride < d
    bad = hexi.make_desc(hexi.HEXI_BF16, 128, 8, 2, -1.0, (1024, 128), (256, 128))
    assert _call_fwd(bad, [(0, 4)], [(0, 4)], good) == hexi.HEXI_EINVAL                   # scale
    assert _call_fwd(d, [(4, 0)], [(0, 4)], good) == hexi.HEXI_EINVAL                     # empty segment
    lib = hexi.load()
    assert lib.hexi_attn_merge_lse(4, 2, 126, 4096, 8192, 12288, 16384, None, 0, None) == hexi.HEXI_EINVAL
    assert lib.hexi_attn_merge_lse(4, 2, 128, 0, 8192, 12288, 16384, None, 0, None) == hexi.HEXI_EINVAL
    assert lib.hexi_attn_merge_lse(0, 2, 128, 4096, 8192, 12288, 16384, None, 0, None) == hexi.HEXI_OK  # nothing to do
    assert hexi.hexi_workspace_bytes(d, 1024, 1024) == 0


def test_workload_geometry():
    w = wl.config(2)
    assert w.q_segs == [(0, 8192), (122880, 8192)] and len(w.chunks) == 8 and w.chunks[0] == w.q_segs
    w = wl.config(3)
    assert w.q_segs == [(32768, 40960)] and len(w.chunks) == 8
    assert [n for ch in w.chunks for _, n in ch][:4] == [20480, 12288, 40960, 24576]
    assert all(n >= 8192 and n % 1024 == 0 for ch in w.chunks for _, n in ch)
    assert wl.config(3).chunks == wl.config(3).chunks  # seeded: reproducible
    w = wl.config(4)
    assert w.q_segs == [(49152, 16384), (458752, 16384)] and w.k_scale == 3.0
    w = wl.config(5)
    assert w.q_segs == [(491520, 32768)] and len(w.chunks) == 32 and w.chunks[15] == [(491520, 32768)]
    m = wl.config(5, shrink=32)
    assert m.lq == 1024 and m.l_tot == 32768 and m.n_q_heads == 8
    x = wl.make_inputs(wl.config(1, shrink=8))
    y = wl.make_inputs(wl.config(1, shrink=8))
    assert all((x[n] == y[n]).all() for n in x) and x["q"].shape == (128, 4, 64)


def test_synthetic_values_are_slices_of_one_global_tensor():
    """A value depends only on (seed, tensor, token, global head, column): every shard of a sequence, whatever its token
    range and head subset, sees the same q / k / v / dO at the same place (so the devices of one plan are consistent)."""
    import torch
    full = wl.global_rows(7, wl.TENSOR_IDS["q"], list(range(6)), 64, [(0, 5000)], torch.float32)
    part = wl.global_rows(7, wl.TENSOR_IDS["q"], [4, 1], 64, [(1000, 37), (2040, 1100), (4999, 1)], torch.float32)
    assert torch.equal(part[:37], full[1000:1037][:, [4, 1]])
    assert torch.equal(part[37:1137], full[2040:3140][:, [4, 1]]) and torch.equal(part[1137:], full[4999:][:, [4, 1]])
    assert not torch.equal(wl.global_rows(7, wl.TENSOR_IDS["k"], [0], 64, [(0, 64)], torch.float32), full[:64, :1])     # another tensor
    assert not torch.equal(wl.global_rows(8, wl.TENSOR_IDS["q"], [0], 64, [(0, 64)], torch.float32), full[:64, :1])     # another seed
    assert abs(float(full.std()) - 1.0) < 0.01 and abs(float(full.mean())) < 0.01
    # two devices of one scheduled plan: common kv heads carry the same K, and a device's q rows are its block of the sequence
    groups, l_group, n_heads = [[0, 1], [2, 3]], [1536, 2560], [2, 1, 1, 2]
    w1 = wl.from_schedule(groups, l_group, n_heads, 1, head_dim=64, q_per_kv=2)
    w3 = wl.from_schedule(groups, l_group, n_heads, 3, head_dim=64, q_per_kv=2)
    assert (w1.q_head_ids, w1.kv_head_ids, w3.q_head_ids, w3.kv_head_ids) == ([2], [1], [1, 2], [0, 1])
    x1, x3 = wl.make_inputs(w1, 3), wl.make_inputs(w3, 3)
    assert torch.equal(x1["k"][:, 0], x3["k"][:, 1]) and torch.equal(x1["v"][:, 0], x3["v"][:, 1])
    q_all = wl.global_rows(3, wl.TENSOR_IDS["q"], [0, 1, 2], 64, [(0, 4096)], torch.bfloat16)
    assert torch.equal(x1["q"], q_all[:1536][:, [2]]) and torch.equal(x3["q"], q_all[1536:][:, [1, 2]])


def test_a2a_argument_validation_without_gpu():
    """hexi_a2a_pack / hexi_a2a_unpack check their tables on the host before anything is launched."""
    lib = hexi.load()
    i32 = ctypes.c_int32

    def call(fn, s=4, n=6, d=128, eb=2, stride=None, counts=(2, 1), heads=(0, 5, 3), ptr=16, ranks=None):
        stride = n * d if stride is None else stride
        c = (i32 * max(1, len(counts)))(*counts)
        h = (i32 * max(1, len(heads)))(*heads)
        return fn(ctypes.c_void_p(ptr), ctypes.c_void_p(ptr), s, n, d, eb, stride, len(counts) if ranks is None else ranks, c, h, None)

    for fn in (lib.hexi_a2a_pack, lib.hexi_a2a_unpack):
        assert call(fn, s=0) == hexi.HEXI_OK                              # nothing to move: no launch
        assert call(fn, counts=(), heads=()) == hexi.HEXI_OK
        assert call(fn, heads=(0, 6, 3)) == hexi.HEXI_EINVAL              # head out of range
        assert call(fn, heads=(0, -1, 3)) == hexi.HEXI_EINVAL
        assert call(fn, counts=(2, -1)) == hexi.HEXI_EINVAL
        assert call(fn, eb=3) == hexi.HEXI_EUNSUPPORTED
        assert call(fn, d=12) == hexi.HEXI_EALIGN                         # 24-byte rows
        assert call(fn, stride=6 * 128 - 8) == hexi.HEXI_EINVAL           # stride smaller than a token
        assert call(fn, ptr=8) == hexi.HEXI_EALIGN
        assert call(fn, ranks=65) == hexi.HEXI_EINVAL
        assert call(fn, n=300, counts=(257,), heads=tuple(range(257))) == hexi.HEXI_EUNSUPPORTED
    assert call(lib.hexi_a2a_unpack, heads=(0, 5, 0)) == hexi.HEXI_EINVAL  # a head written twice
    assert b"twice" in lib.hexi_last_error()
