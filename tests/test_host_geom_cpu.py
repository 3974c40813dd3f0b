"""The integer helpers that the kernels themselves use to decide visibility (seg_pos_of_row, seg_rows_le) and the
dK/dV launcher's head-run builder, compiled for the host alone and compared bit for bit with the oracle's position
walk and with plain Python definitions.  (hexi_shard_mask's outputs feed no kernel; these functions do.)"""
import os
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def geom_binary(tmp_path_factory):
    hipcc = "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    exe = str(tmp_path_factory.mktemp("geom") / "geom_check")
    subprocess.check_call([hipcc, "-O1", "-std=c++17", "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
                           "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_2605_07569_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host", "geom_check.cpp"), "-o", exe])
    return exe


def _ask(exe, lines):
    return subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, check=True).stdout.strip().splitlines()


def _random_segs(rng, n_seg, max_len, max_gap):
    out, cur = [], int(rng.integers(0, max_gap + 1))
    for _ in range(n_seg):
        ln = int(rng.integers(1, max_len + 1))
        out.append((cur, ln))
        cur += ln + int(rng.integers(0, max_gap + 1))
    return out


def test_row_positions_and_visible_row_counts_match_the_oracle(geom_binary):
    rng = np.random.default_rng(31)
    cases = [[(0, 1)], [(5, 1), (6, 1)], [(0, 8192), (122880, 8192)], [(3, 4), (7, 2), (100, 1)]]
    cases += [_random_segs(rng, int(rng.integers(1, 17)), 200, 150) for _ in range(40)]
    lines, queries = [], []
    for segs in cases:
        lo, hi = segs[0][0], segs[-1][0] + segs[-1][1]
        ps = sorted(set([-1, 0, lo - 1, lo, hi - 1, hi, hi + 7] + [s - 1 for s, _ in segs] + [s + n - 1 for s, n in segs] +
                        [s + n for s, n in segs] + [int(x) for x in rng.integers(0, hi + 2, size=25)]))
        queries.append(ps)
        lines.append("seg %d %s %s" % (len(segs), " ".join(f"{s} {n}" for s, n in segs), " ".join(str(p) for p in ps)))
    for segs, ps, out in zip(cases, queries, _ask(geom_binary, lines)):
        left, right = out.split("|")
        pos = oracle.positions(segs)
        assert np.array_equal(np.array(left.split(), dtype=np.int64), pos), segs
        # rows whose position is <= p: counted on the oracle's position list
        want = [int(np.sum(pos <= p)) for p in ps]
        assert [int(x) for x in right.split()] == want, segs


def test_head_runs_cover_every_head_once(geom_binary):
    rng = np.random.default_rng(5)
    cases = [(128, 1, 128, [0] * 128), (128, 1, 127, [0] * 128), (128, 1, 1, [0] * 128), (8, 3, 3, [0, 1, 0, 0, 2, 0, 1, 0]),
             (24, 8, 3, [h // 3 for h in range(24)]), (6, 3, 2, [2, 0, 1, 0, 2, 2])]
    for _ in range(30):
        nkv = int(rng.integers(1, 9))
        nq = int(rng.integers(nkv, 129))
        cases.append((nq, nkv, int(rng.integers(1, 130)), [int(x) for x in rng.integers(0, nkv, size=nq)]))
    lines = ["runs %d %d %d %s" % (nq, nkv, rl, " ".join(map(str, m))) for nq, nkv, rl, m in cases]
    for (nq, nkv, rl, m), out in zip(cases, _ask(geom_binary, lines)):
        tok = out.split()
        shared, n_runs, runs = int(tok[0]), int(tok[1]), tok[2:]
        assert len(runs) == n_runs
        # definition: the heads of each kv head, in head order, cut into consecutive runs of at most rl heads
        want = []
        for kh in range(nkv):
            hs = [h for h in range(nq) if m[h] == kh]
            want += [hs[i:i + rl] for i in range(0, len(hs), rl)]
        got = []
        for r in runs:
            first, ln, heads = r.split(":")
            hs = [int(x) for x in heads.split(",") if x]
            assert hs[0] == int(first) and len(hs) == int(ln)
            got.append(hs)
        assert sorted(got) == sorted(want), (nq, nkv, rl)
        assert shared == int(any(sum(1 for g in got if m[g[0]] == kh) > 1 for kh in range(nkv)))
    # the single run of 128 heads: its length must not wrap
    assert _ask(geom_binary, [lines[0]])[0].split()[2].startswith("0:128:")
