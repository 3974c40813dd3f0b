"""Host logic of the kernel launchers: the split of a launch's work units over the 8 XCDs (contiguous unit
ranges of nearly equal estimated work).  The helper is compiled for the host alone and fed weight lists."""
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def split_binary(tmp_path_factory):
    hipcc = "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    exe = str(tmp_path_factory.mktemp("split") / "split_check")
    subprocess.check_call([hipcc, "-O1", "-std=c++17", "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
                           "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_2605_07569_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host", "split_check.cpp"), "-o", exe])
    return exe


def _split(exe, lists):
    text = "\n".join(" ".join(repr(float(x)) for x in w) for w in lists) + "\n"
    out = subprocess.run([exe], input=text, capture_output=True, text=True, check=True).stdout.strip().splitlines()
    return [[int(t) for t in line.split()] for line in out]


def test_ranges_partition_the_units_and_balance_the_work(split_binary):
    rng = np.random.default_rng(8)
    lists = [np.ones(1920), np.ones(5), np.ones(1), np.ones(8), np.ones(1027)]
    # causal launch: 12 heads x 160 q tiles, a head's units falling linearly in length (the diagonal chunk of the
    # asymmetric configuration), plus the constant per-unit overhead
    tri = np.concatenate([np.arange(160, 0, -1) * 2.5 + 6.0 for _ in range(12)])
    lists += [tri, rng.uniform(0.25, 700.0, size=3000), np.concatenate([np.full(700, 0.25), np.full(68, 262.0)])]
    for w, row in zip(lists, _split(split_binary, lists)):
        start, grid = row[:9], row[9]
        n = len(w)
        assert start[0] == 0 and start[8] == n and all(a <= b for a, b in zip(start, start[1:]))
        counts = np.diff(start)
        assert grid == 8 * counts.max()
        loads = np.array([w[a:b].sum() for a, b in zip(start, start[1:])])
        # a range ends with the unit that carries its cumulative share over x/8 of the total: no range exceeds the
        # mean by more than the heaviest unit
        assert loads.max() <= w.sum() / 8 + w.max() + 1e-9
        if np.all(w == w[0]):
            assert counts.max() - counts.min() <= 1
    # the triangle case really is balanced far better than equal counts would be
    tri_start = _split(split_binary, [tri])[0][:9]
    loads = np.array([tri[a:b].sum() for a, b in zip(tri_start, tri_start[1:])])
    equal = np.array([tri[240 * x:240 * (x + 1)].sum() for x in range(8)])
    assert loads.max() / loads.mean() < 1.02 < 1.15 < equal.max() / equal.mean()
