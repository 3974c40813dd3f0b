"""Thin ctypes binding over libhexi_attn.so (the C ABI of include/hexi_attn.h).

Argument marshalling only: every step of the attention path runs in the library's HIP kernels.
Tensors are torch tensors used as device-memory handles (``data_ptr()``); the stream is torch's
current HIP stream unless given.  There is no CPU fallback: if the library has not been built,
loading raises.
"""
import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

HEXI_OK = 0
HEXI_EINVAL, HEXI_EUNSUPPORTED, HEXI_EALIGN, HEXI_EWORKSPACE, HEXI_EHIP, HEXI_EINFEASIBLE = -1, -2, -3, -4, -5, -6
HEXI_BF16, HEXI_F32 = 0, 1
HEXI_ACCUMULATE, HEXI_COMPUTE_DELTA, HEXI_SKIP_DQ, HEXI_SKIP_DKDV = 1, 2, 4, 8
HEXI_TILE_EMPTY, HEXI_TILE_FULL, HEXI_TILE_PARTIAL = 0, 1, 2
HEXI_MAX_SEGS = 16

EXPORTS = ("hexi_shard_mask", "hexi_attn_fwd_chunk", "hexi_attn_merge_lse", "hexi_attn_bwd_chunk",
           "hexi_a2a_pack", "hexi_a2a_unpack", "hexi_sched_cost", "hexi_sched_solve", "hexi_set_dkdv_run_len", "hexi_workspace_bytes", "hexi_last_error", "hexi_version")

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhexi_attn.so")
PROBE_LIB_PATH = os.path.join(_HERE, "libhexi_probe.so")     # include/hexi_probe.h: the benchmark's MFMA rate probe
PROBE_EXPORTS = ("hexi_mfma_probe",)
_lib = None
_probe_lib = None


class HexiError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"hexi error {code}: {msg}")
        self.code = code


class hexi_seg(ctypes.Structure):
    _fields_ = [("start", ctypes.c_int64), ("len", ctypes.c_int64)]


class hexi_range(ctypes.Structure):
    _fields_ = [("n_segs", ctypes.c_int32), ("segs", ctypes.POINTER(hexi_seg))]


class hexi_attn_desc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("kv_of_q", ctypes.POINTER(ctypes.c_int32)), ("softmax_scale", ctypes.c_float),
                ("q_stride_tok", ctypes.c_int64), ("q_stride_head", ctypes.c_int64),
                ("kv_stride_tok", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64)]


def load():
    """Loads the in-tree library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_07569_amd.build` "
                           "(hipcc, gfx950); there is no CPU fallback")
    import torch  # noqa: F401  (loads the HIP runtime the library binds to)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32
    rp, dp = ctypes.POINTER(hexi_range), ctypes.POINTER(hexi_attn_desc)
    lib.hexi_shard_mask.argtypes = [rp, rp, i32, i32, vp, vp, vp, ctypes.POINTER(i64)]
    lib.hexi_shard_mask.restype = ctypes.c_int
    lib.hexi_attn_fwd_chunk.argtypes = [dp, rp, rp, vp, vp, vp, vp, vp, u32, vp, ctypes.c_size_t, vp]
    lib.hexi_attn_fwd_chunk.restype = ctypes.c_int
    lib.hexi_attn_merge_lse.argtypes = [i64, i32, i32, vp, vp, vp, vp, vp, i32, vp]
    lib.hexi_attn_merge_lse.restype = ctypes.c_int
    lib.hexi_attn_bwd_chunk.argtypes = [dp, rp, rp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, u32, vp, ctypes.c_size_t, vp]
    lib.hexi_attn_bwd_chunk.restype = ctypes.c_int
    i32p = ctypes.POINTER(i32)
    lib.hexi_a2a_pack.argtypes = [vp, vp, i64, i32, i32, i32, i64, i32, i32p, i32p, vp]
    lib.hexi_a2a_pack.restype = ctypes.c_int
    lib.hexi_a2a_unpack.argtypes = [vp, vp, i64, i32, i32, i32, i64, i32, i32p, i32p, vp]
    lib.hexi_a2a_unpack.restype = ctypes.c_int
    lib.hexi_sched_cost.argtypes = [vp, vp, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    lib.hexi_sched_cost.restype = ctypes.c_int
    lib.hexi_sched_solve.argtypes = [vp, vp, vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.hexi_sched_solve.restype = ctypes.c_int
    lib.hexi_set_dkdv_run_len.argtypes = [i32]
    lib.hexi_set_dkdv_run_len.restype = i32
    lib.hexi_workspace_bytes.argtypes = [dp, i64, i64]
    lib.hexi_workspace_bytes.restype = ctypes.c_size_t
    lib.hexi_last_error.restype = ctypes.c_char_p
    lib.hexi_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def load_probe():
    """Loads the benchmark's measurement-aid library (not part of the attention interface)."""
    global _probe_lib
    if _probe_lib is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise RuntimeError(f"{PROBE_LIB_PATH} is missing: build it with `python -m paper_2605_07569_amd.build`")
        import torch  # noqa: F401
        lib = ctypes.CDLL(PROBE_LIB_PATH)
        lib.hexi_mfma_probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
        lib.hexi_mfma_probe.restype = ctypes.c_int
        _probe_lib = lib
    return _probe_lib


def _check(rc):
    if rc != HEXI_OK:
        raise HexiError(rc, load().hexi_last_error().decode())


def make_range(segs: Sequence[Tuple[int, int]]):
    """[(start, len), ...] -> (hexi_range, keepalive)."""
    arr = (hexi_seg * max(1, len(segs)))(*[hexi_seg(int(s), int(n)) for s, n in segs])
    return hexi_range(len(segs), arr), arr


def make_desc(dtype, head_dim, n_q_heads, n_kv_heads, softmax_scale, q_strides, kv_strides, kv_of_q=None):
    """q_strides / kv_strides: (token stride, head stride) in elements."""
    keep = None
    ptr = ctypes.POINTER(ctypes.c_int32)()
    if kv_of_q is not None:
        keep = (ctypes.c_int32 * len(kv_of_q))(*[int(x) for x in kv_of_q])
        ptr = ctypes.cast(keep, ctypes.POINTER(ctypes.c_int32))
    d = hexi_attn_desc(int(dtype), int(head_dim), int(n_q_heads), int(n_kv_heads), ptr, float(softmax_scale),
                       int(q_strides[0]), int(q_strides[1]), int(kv_strides[0]), int(kv_strides[1]))
    d._keep = keep
    return d


def desc_for(q, k, softmax_scale, kv_of_q=None):
    """Descriptor for torch tensors q [Lq, nq, d] and k [Lc, nkv, d] (d contiguous)."""
    import torch
    assert q.dim() == 3 and k.dim() == 3 and q.stride(2) == 1 and k.stride(2) == 1
    dt = {torch.bfloat16: HEXI_BF16, torch.float32: HEXI_F32}[q.dtype]
    return make_desc(dt, q.shape[2], q.shape[1], k.shape[1], softmax_scale,
                     (q.stride(0), q.stride(1)), (k.stride(0), k.stride(1)), kv_of_q)


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return ctypes.c_void_p(int(stream))


def hexi_version():
    return load().hexi_version().decode()


def hexi_last_error():
    return load().hexi_last_error().decode()


def hexi_shard_mask(q_segs, kv_segs, tile_m=0, tile_n=0, want_pos=True, want_classes=True):
    """Host bookkeeping -> dict(q_pos, kv_pos (int32 numpy), tile_class (uint8 [nm, nn]), n_pairs)."""
    lib = load()
    qr, _k1 = make_range(q_segs)
    kr, _k2 = make_range(kv_segs)
    lq, lc = sum(int(n) for _, n in q_segs), sum(int(n) for _, n in kv_segs)
    q_pos = np.empty(max(lq, 0), dtype=np.int32) if want_pos else None
    kv_pos = np.empty(max(lc, 0), dtype=np.int32) if want_pos else None
    cls = None
    if want_classes and tile_m > 0 and tile_n > 0:
        cls = np.empty((-(-lq // tile_m), -(-lc // tile_n)), dtype=np.uint8)
    n_pairs = ctypes.c_int64(0)
    rc = lib.hexi_shard_mask(ctypes.byref(qr), ctypes.byref(kr), tile_m, tile_n,
                             None if q_pos is None else q_pos.ctypes.data_as(ctypes.c_void_p),
                             None if kv_pos is None else kv_pos.ctypes.data_as(ctypes.c_void_p),
                             None if cls is None else cls.ctypes.data_as(ctypes.c_void_p),
                             ctypes.byref(n_pairs))
    _check(rc)
    return dict(q_pos=q_pos, kv_pos=kv_pos, tile_class=cls, n_pairs=int(n_pairs.value))


def hexi_attn_fwd_chunk(desc, q_segs, kv_segs, q, k, v, o, lse, flags=0, workspace=None, stream=None):
    qr, _k1 = make_range(q_segs)
    kr, _k2 = make_range(kv_segs)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().hexi_attn_fwd_chunk(ctypes.byref(desc), ctypes.byref(qr), ctypes.byref(kr), _ptr(q), _ptr(k), _ptr(v),
                                      _ptr(o), _ptr(lse), flags, _ptr(workspace), ws_bytes, _stream(stream)))


def hexi_attn_merge_lse(o_acc, lse_acc, o_part, lse_part, o_final=None, stream=None):
    import torch
    n_rows, nq, d = o_acc.shape
    fdt = HEXI_F32
    if o_final is not None:
        fdt = {torch.bfloat16: HEXI_BF16, torch.float32: HEXI_F32}[o_final.dtype]
    _check(load().hexi_attn_merge_lse(n_rows, nq, d, _ptr(o_acc), _ptr(lse_acc), _ptr(o_part), _ptr(lse_part),
                                      _ptr(o_final), fdt, _stream(stream)))


def hexi_attn_bwd_chunk(desc, q_segs, kv_segs, q, k, v, o, d_o, lse, delta, dq_acc, dk, dv, flags=0,
                        workspace=None, stream=None):
    qr, _k1 = make_range(q_segs)
    kr, _k2 = make_range(kv_segs)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().hexi_attn_bwd_chunk(ctypes.byref(desc), ctypes.byref(qr), ctypes.byref(kr), _ptr(q), _ptr(k), _ptr(v),
                                      _ptr(o), _ptr(d_o), _ptr(lse), _ptr(delta), _ptr(dq_acc), _ptr(dk), _ptr(dv),
                                      flags, _ptr(workspace), ws_bytes, _stream(stream)))


def hexi_workspace_bytes(desc, lq, lc):
    return int(load().hexi_workspace_bytes(ctypes.byref(desc), lq, lc))


def _head_tables(head_lists):
    counts = (ctypes.c_int32 * max(1, len(head_lists)))(*[len(h) for h in head_lists])
    flat = [int(h) for heads in head_lists for h in heads]
    heads = (ctypes.c_int32 * max(1, len(flat)))(*flat)
    return counts, heads


def hexi_a2a_pack(x, packed, head_lists, stream=None):
    """x: [s, n_heads_total, d] (token stride may exceed a token); packed: contiguous 1-D buffer of the same
    dtype with sum(len(l)) * s * d elements; head_lists: one list of head indices per destination rank."""
    s, n, d = x.shape
    counts, heads = _head_tables(head_lists)
    _check(load().hexi_a2a_pack(_ptr(x), _ptr(packed), s, n, d, x.element_size(), x.stride(0), len(head_lists), counts, heads,
                                _stream(stream)))


def hexi_a2a_unpack(packed, y, head_lists, stream=None):
    """Inverse of hexi_a2a_pack: scatters the per-rank parts of `packed` into y [s, n_heads_total, d]."""
    s, n, d = y.shape
    counts, heads = _head_tables(head_lists)
    _check(load().hexi_a2a_unpack(_ptr(packed), _ptr(y), s, n, d, y.element_size(), y.stride(0), len(head_lists), counts, heads,
                                  _stream(stream)))


class _Cluster(ctypes.Structure):
    _fields_ = [("n_devices", ctypes.c_int32)] + [(k, ctypes.POINTER(ctypes.c_double)) for k in ("c", "b", "m", "m_static", "alpha", "bw")]


class _Model(ctypes.Structure):
    _fields_ = [("l_tot", ctypes.c_int64), ("batch", ctypes.c_int32), ("hidden", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_heads", ctypes.c_int32), ("dtype_bytes", ctypes.c_int32), ("gamma_act", ctypes.c_double)]


class _SchedOpts(ctypes.Structure):
    _fields_ = [("m1", ctypes.c_int32), ("m2", ctypes.c_int32), ("i_max", ctypes.c_int32), ("token_quantum", ctypes.c_int32),
                ("gap_ratio", ctypes.c_double), ("perturb", ctypes.c_double), ("move_tokens", ctypes.c_int64)]


class _Schedule(ctypes.Structure):
    _fields_ = [("n_groups", ctypes.c_int32), ("group_of", ctypes.POINTER(ctypes.c_int32)), ("l_group", ctypes.POINTER(ctypes.c_int64)),
                ("s_pre", ctypes.POINTER(ctypes.c_int64)), ("n_heads", ctypes.POINTER(ctypes.c_int32))]


def _cluster_struct(c, b, m, m_static, alpha, bw):
    n = len(c)
    arrs = [np.ascontiguousarray(a, dtype=np.float64) for a in (c, b, m, m_static, np.asarray(alpha).reshape(-1), np.asarray(bw).reshape(-1))]
    st = _Cluster(n, *[a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) for a in arrs])
    return st, arrs


def _model_struct(l_tot, batch, hidden, head_dim, n_heads, dtype_bytes, gamma_act=2.0):
    return _Model(l_tot, batch, hidden, head_dim, n_heads, dtype_bytes, gamma_act)


def hexi_sched_cost(cluster, model, groups, l_group, s_pre, n_heads):
    """cluster: dict(c, b, m, m_static, alpha, bw); model: dict(l_tot, batch, hidden, head_dim, n_heads, dtype_bytes[, gamma_act]);
    groups: list of device lists in ring order.  Returns (T_blk, max T_nonattn, max T_A2A, sum T_step, feasible)."""
    cs, keep = _cluster_struct(**cluster)
    ms = _model_struct(**model)
    n = cs.n_devices
    group_of = np.full(n, -1, dtype=np.int32)
    for k, g in enumerate(groups):
        for d in g:
            group_of[d] = k
    lg = np.zeros(n, dtype=np.int64)
    lg[:len(groups)] = l_group
    sp, nh = np.ascontiguousarray(s_pre, dtype=np.int64), np.ascontiguousarray(n_heads, dtype=np.int32)
    sch = _Schedule(len(groups), group_of.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), lg.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                    sp.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), nh.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    terms = (ctypes.c_double * 4)()
    feas = ctypes.c_int32(0)
    _check(load().hexi_sched_cost(ctypes.byref(cs), ctypes.byref(ms), ctypes.byref(sch), terms, ctypes.byref(feas)))
    return terms[0], terms[1], terms[2], terms[3], bool(feas.value)


def hexi_sched_solve(cluster, model, **opts):
    """Returns dict(groups, l_group, s_pre, n_heads, cost).  opts: m1, m2, i_max, token_quantum, gap_ratio, perturb, move_tokens."""
    cs, keep = _cluster_struct(**cluster)
    ms = _model_struct(**model)
    n = cs.n_devices
    o = _SchedOpts(opts.get("m1", 0), opts.get("m2", 0), opts.get("i_max", 0), opts.get("token_quantum", 0),
                   opts.get("gap_ratio", 0.0), opts.get("perturb", 0.0), opts.get("move_tokens", 0))
    group_of, lg = np.zeros(n, dtype=np.int32), np.zeros(n, dtype=np.int64)
    sp, nh = np.zeros(n, dtype=np.int64), np.zeros(n, dtype=np.int32)
    sch = _Schedule(0, group_of.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), lg.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                    sp.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), nh.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    cost = ctypes.c_double(0.0)
    _check(load().hexi_sched_solve(ctypes.byref(cs), ctypes.byref(ms), ctypes.byref(o), ctypes.byref(sch), ctypes.byref(cost)))
    groups = [[d for d in range(n) if group_of[d] == k] for k in range(sch.n_groups)]
    return dict(groups=groups, l_group=[int(x) for x in lg[:sch.n_groups]], s_pre=[int(x) for x in sp], n_heads=[int(x) for x in nh],
                cost=cost.value)


def hexi_set_dkdv_run_len(run_len):
    """0: the library chooses per call; n >= 1: at most n q heads per dK/dV workgroup run.  Returns the previous value."""
    return int(load().hexi_set_dkdv_run_len(int(run_len)))


def hexi_mfma_probe(operands, sink, iters, stream=None):
    """operands: 65536 bytes of bf16 on the device; sink: float32[256 * 512] on the device."""
    rc = load_probe().hexi_mfma_probe(_ptr(operands), _ptr(sink), int(iters), _stream(stream))
    if rc != 0:
        raise HexiError(rc, "hexi_mfma_probe refused its arguments or the launch")

