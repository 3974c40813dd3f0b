"""Builds libhexi_attn.so (gfx950) in-tree with hipcc.  `python -m paper_2605_07569_amd.build`."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhexi_attn.so")
PROBE_LIB = os.path.join(HERE, "libhexi_probe.so")      # the benchmark's measurement aid (include/hexi_probe.h)
EXPORT_MAP = os.path.join(CSRC, "hexi_exports.map")     # only hexi_* symbols leave the libraries
SOURCES = ["hexi_api.hip", "hexi_sched.cpp", "hexi_misc.hip", "hexi_a2a.hip", "hexi_f32.hip", "hexi_bf16_fwd.hip", "hexi_bf16_bwd.hip", "hexi_bf16_bwd_dq.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-munsafe-fp-atomics", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-inline-asm",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc():
    for p in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.exists(p) or p == "hipcc":
            return p


def _compile(src):
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    if src.endswith(".cpp"):   # host-only code: no device pass, no fused multiply-adds (results must not depend on them)
        cmd = [_hipcc(), "-O2", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-ffp-contract=off",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "c++", "-c", os.path.join(CSRC, src), "-o", obj]
    else:
        cmd = [_hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose=True):
    with ThreadPoolExecutor(max_workers=len(SOURCES) + 1) as ex:
        objs = list(ex.map(_compile, SOURCES + ["hexi_probe.hip"]))
    link = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-Wl,--version-script=" + EXPORT_MAP]
    subprocess.check_call(link + ["-o", LIB] + objs[:-1])
    subprocess.check_call(link + ["-o", PROBE_LIB] + objs[-1:])
    if verbose:
        print("built", LIB, "and", PROBE_LIB)
    return LIB


if __name__ == "__main__":
    build()
