"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer: the fp64 oracle (oracle/hexi_oracle.c), the
library's host scheduler (csrc/hexi_sched.cpp) and the integer helpers of the kernels and launchers
(csrc/hexi_internal.h) are compiled for the host with -fsanitize=address,undefined -fno-sanitize-recover and run
once on small inputs; the runs must end cleanly and give the same answers as the ordinary builds."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from paper_2605_07569_amd import hexi
from sched_util import cluster_arrays, model_args

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:exitcode=97", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1:exitcode=98")


def _need(tool):
    if shutil.which(tool) is None:
        pytest.skip(f"{tool} not available")


def _run(cmd, text=""):
    r = subprocess.run(cmd, input=text, capture_output=True, text=True, env=ENV)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr and "LeakSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    _need("gcc")
    exe = str(tmp_path / "san_oracle")
    subprocess.check_call(["gcc", "-std=c99", "-fopenmp"] + SAN + [os.path.join(ROOT, "tests", "host", "sanitize_oracle.c"), "-o", exe, "-lm"])
    out = _run([exe])
    assert out.startswith("ok "), out
    # the same driver without the sanitizers gives the same checksum (they do not change the arithmetic)
    plain = str(tmp_path / "plain_oracle")
    subprocess.check_call(["gcc", "-std=c99", "-fopenmp", "-O1", os.path.join(ROOT, "tests", "host", "sanitize_oracle.c"), "-o", plain, "-lm"])
    assert float(_run([plain]).split()[1]) == pytest.approx(float(out.split()[1]), rel=1e-12)


def test_host_scheduler_under_asan_ubsan_matches_the_library(tmp_path):
    _need("g++")
    exe = str(tmp_path / "san_sched")
    subprocess.check_call(["g++", "-std=c++17", "-pthread", "-ffp-contract=off"] + SAN +
                          ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2605_07569_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host", "sanitize_sched.cpp"), "-o", exe])
    cases = [([("h100", 2), ("a100", 2)], model_args(l_tot=16384, n_heads=8, hidden=1024), dict(m1=8, m2=4, i_max=20)),
             ([("h100", 2), ("a100", 3), ("a800", 2)], model_args(l_tot=32768, n_heads=40, hidden=5120), dict(m2=6, i_max=30)),
             ([("a100", 1)], model_args(l_tot=4096, n_heads=8), dict())]
    for nodes, margs, opts in cases:
        arr = cluster_arrays(nodes, jitter_seed=7)
        n = len(arr["c"])
        nums = [n] + arr["c"] + arr["b"] + arr["m"] + arr["m_static"] + [x for r in arr["alpha"] for x in r] + [x for r in arr["bw"] for x in r]
        nums += [margs["l_tot"], margs["batch"], margs["hidden"], margs["head_dim"], margs["n_heads"], margs["dtype_bytes"], 2.0]
        nums += [opts.get("m1", 0), opts.get("m2", 0), opts.get("i_max", 0), 0, 0]
        out = _run([exe], " ".join(repr(x) for x in nums) + "\n").split("\n")
        want = hexi.hexi_sched_solve(arr, margs, **opts)
        k = int(out[0].split()[1])
        rows = [tuple(int(x) for x in line.split()) for line in out[1:1 + n]]
        assert k == len(want["groups"])
        assert [r[0] for r in rows] == [next(i for i, g in enumerate(want["groups"]) if d in g) for d in range(n)]
        assert [r[1] for r in rows] == want["s_pre"] and [r[2] for r in rows] == want["n_heads"]
        assert [int(line.split()[1]) for line in out[1 + n:1 + n + k]] == want["l_group"]
        tail = out[1 + n + k].split()
        assert float(tail[1]) == pytest.approx(want["cost"], rel=1e-12) and tail[-1] == "1"
        assert float(tail[3]) == pytest.approx(float(tail[1]), rel=1e-12)


def test_kernel_host_helpers_under_asan_ubsan(tmp_path):
    """seg_pos_of_row / seg_rows_le, the head-run builder and the XCD work split, in the sanitized build, on the
    cases of their own tests (16-segment tables, 128 heads in one run, a thousand work units)."""
    _need("g++")
    inc = ["-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2605_07569_amd", "csrc")]
    if not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"):
        pytest.skip("HIP headers not available")
    hipcc = "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    geom, split = str(tmp_path / "geom"), str(tmp_path / "split")
    for src, exe in (("geom_check.cpp", geom), ("split_check.cpp", split)):
        # host-only translation units: no device pass, and the sanitizers stay off any GPU code
        subprocess.check_call([hipcc, "-std=c++17", "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-fno-gpu-sanitize"] + SAN + inc + [os.path.join(ROOT, "tests", "host", src), "-o", exe])
    rng = np.random.default_rng(3)
    lines = []
    for _ in range(20):
        n = int(rng.integers(1, 17))
        cur, segs = int(rng.integers(0, 50)), []
        for _ in range(n):
            ln = int(rng.integers(1, 300))
            segs.append((cur, ln))
            cur += ln + int(rng.integers(0, 100))
        lines.append("seg %d %s %s" % (n, " ".join(f"{s} {l}" for s, l in segs), " ".join(str(int(p)) for p in rng.integers(-2, cur + 3, size=30))))
    lines.append("runs 128 1 128 " + " ".join(["0"] * 128))
    lines.append("runs 128 8 5 " + " ".join(str(int(x)) for x in rng.integers(0, 8, size=128)))
    assert len(_run([geom], "\n".join(lines) + "\n").strip().splitlines()) == len(lines)
    weights = [np.ones(1920), rng.uniform(0.25, 700.0, size=3000), np.ones(1)]
    out = _run([split], "\n".join(" ".join(repr(float(x)) for x in w) for w in weights) + "\n").strip().splitlines()
    assert len(out) == len(weights)
