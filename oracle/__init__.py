"""fp64 CPU oracle for one device's share of context-parallel causal attention.

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It is a ctypes wrapper over
``hexi_oracle.c`` (plain C, fp64, OpenMP), which writes out the textbook definition of causal
softmax attention and its gradients for the step shape of HexiSeq App. A.4 (Eq. 10-11).  It imports
nothing from the HIP package and shares no code with it.

Arrays are numpy float64, C-contiguous: q/o/d_o/dq ``[Lq, nq, d]``; k/v/dk/dv ``[Lk, nkv, d]``;
lse/delta ``[nq, Lq]``; positions int64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hexi_oracle.c")
_LIB = os.path.join(_HERE, "libhexi_oracle.so")
_lib = None


def build(force=True):
    """Compile hexi_oracle.c with gcc (baseline x86-64 code so it runs on any host)."""
    if force or not os.path.exists(_LIB):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        lib.oracle_mask_bruteforce.restype = ctypes.c_int64
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads():
    return int(_load().oracle_num_threads())


def _kv_map(kv_of_q, nq, nkv):
    if kv_of_q is None:
        assert nq % nkv == 0
        kv_of_q = np.arange(nq) // (nq // nkv)
    m = np.ascontiguousarray(kv_of_q, dtype=np.int32)
    assert m.shape == (nq,) and m.min() >= 0 and m.max() < nkv
    return m


def positions(segs):
    """Global token positions of a shard given as [(start, len), ...] packed back to back."""
    segs = [(int(s), int(n)) for s, n in segs]
    total = sum(n for _, n in segs)
    pos = np.empty(total, dtype=np.int64)
    st = _i64([s for s, _ in segs])
    ln = _i64([n for _, n in segs])
    _load().oracle_positions(ctypes.c_int(len(segs)), _p(st), _p(ln), _p(pos))
    return pos


def attn_fwd(q, q_pos, k, v, kv_pos, scale, kv_of_q=None):
    """Exact causal attention of the given rows over the given keys -> (o [Lq,nq,d], lse [nq,Lq])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    q_pos, kv_pos = _i64(q_pos), _i64(kv_pos)
    Lq, nq, d = q.shape
    Lk, nkv, _ = k.shape
    assert k.shape == v.shape and k.shape[2] == d and q_pos.shape == (Lq,) and kv_pos.shape == (Lk,)
    m = _kv_map(kv_of_q, nq, nkv)
    o = np.empty_like(q)
    lse = np.empty((nq, Lq), dtype=np.float64)
    _load().oracle_attn_fwd(ctypes.c_int64(Lq), ctypes.c_int(nq), ctypes.c_int(d), _p(q), _p(q_pos),
                            ctypes.c_int64(Lk), ctypes.c_int(nkv), _p(k), _p(v), _p(kv_pos), _p(m),
                            ctypes.c_double(scale), _p(o), _p(lse))
    return o, lse


def attn_bwd(q, q_pos, k, v, kv_pos, d_o, scale, kv_of_q=None):
    """Gradients of sum <O, dO> -> dict(dq, dk, dv, lse, delta); dk/dv from these q rows only."""
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    q_pos, kv_pos = _i64(q_pos), _i64(kv_pos)
    Lq, nq, d = q.shape
    Lk, nkv, _ = k.shape
    assert k.shape == v.shape and d_o.shape == q.shape and k.shape[2] == d
    m = _kv_map(kv_of_q, nq, nkv)
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    lse = np.empty((nq, Lq), dtype=np.float64)
    delta = np.empty((nq, Lq), dtype=np.float64)
    _load().oracle_attn_bwd(ctypes.c_int64(Lq), ctypes.c_int(nq), ctypes.c_int(d), _p(q), _p(q_pos),
                            ctypes.c_int64(Lk), ctypes.c_int(nkv), _p(k), _p(v), _p(kv_pos), _p(m),
                            ctypes.c_double(scale), _p(d_o), _p(dq), _p(dk), _p(dv), _p(lse), _p(delta))
    return dict(dq=dq, dk=dk, dv=dv, lse=lse, delta=delta)


def delta(o, d_o):
    o, d_o = _f64(o), _f64(d_o)
    Lq, nq, d = o.shape
    out = np.empty((nq, Lq), dtype=np.float64)
    _load().oracle_delta(ctypes.c_int64(Lq), ctypes.c_int(nq), ctypes.c_int(d), _p(o), _p(d_o), _p(out))
    return out


def merge(o_a, lse_a, o_b, lse_b):
    """Two-term log-sum-exp merge of normalised partial results -> (o, lse)."""
    o_a, o_b, lse_a, lse_b = _f64(o_a), _f64(o_b), _f64(lse_a), _f64(lse_b)
    n, nq, d = o_a.shape
    assert o_b.shape == o_a.shape and lse_a.shape == (nq, n) and lse_b.shape == (nq, n)
    o = np.empty_like(o_a)
    lse = np.empty_like(lse_a)
    _load().oracle_merge(ctypes.c_int64(n), ctypes.c_int(nq), ctypes.c_int(d), _p(o_a), _p(lse_a),
                         _p(o_b), _p(lse_b), _p(o), _p(lse))
    return o, lse


def mask_bruteforce(q_pos, kv_pos, tile_m, tile_n):
    """Pair-by-pair tile classes (0 EMPTY, 1 FULL, 2 PARTIAL) and the visible-pair count."""
    q_pos, kv_pos = _i64(q_pos), _i64(kv_pos)
    nm = -(-len(q_pos) // tile_m)
    nn = -(-len(kv_pos) // tile_n)
    cls = np.zeros((nm, nn), dtype=np.uint8)
    n = _load().oracle_mask_bruteforce(ctypes.c_int64(len(q_pos)), _p(q_pos), ctypes.c_int64(len(kv_pos)),
                                       _p(kv_pos), ctypes.c_int(tile_m), ctypes.c_int(tile_n), _p(cls))
    return cls, int(n)
