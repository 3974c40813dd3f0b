#!/usr/bin/env python3
"""Benchmark of the chunked-ring attention hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic shard: forward replay of the KV chunk
list (fwd_chunk with the fused LSE merge), Delta, backward replay (bwd_chunk per chunk).  Inputs are
resident in HBM before the timed region.  Prints one JSON line: fwd+bwd TFLOP/s counted on unmasked
(query, key) pairs only (4*d forward + 10*d backward flops per pair per q head) on the headline
workload -- configuration 4, the largest single-GPU shard (8B-like, 512K tokens, 16 chunks) -- the
roofline position of the dominant kernel (the bf16 dK/dV backward kernel) measured with HIP events
around its launches inside the timed region, the other bf16 configurations (2, 3, 5) timed the same
way over fewer steps under "other_workloads", the zigzag configurations replayed with contiguous
chunks under "contiguous_chunk_replay", and the fp64 CPU oracle timed on a bounded sample of the
headline workload as a reported baseline.  Progress lines go to stderr.
"""
import argparse
import json
import sys
import time

import torch

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16 MFMA peak: 256 CU x 2.4 GHz x 4096 flop/clk/CU
# HBM bytes per launch of the dominant kernel (the dK/dV kernel on a remote chunk) from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of `bench.py --workload N --only-headline --copy-calibration` (see profiles/): fetched + written,
# each scaled by what the same counter reads for a 1 GiB device copy.
MEASURED_TRAFFIC_BYTES = {
    "cfg2_3b_zigzag": 0.676e9,    # <128, false>: 496 MB fetched + 180 MB written
    "cfg3_8b_asym": 1.18e9,       # <128, true>, the 12K-key chunk: 1020 MB + 160 MB
    "cfg4_8b_long": 3.22e9,       # <128, true>: 2480 MB + 738 MB
    "cfg5_70b_hp": 1.61e9,        # <128, true>: 1241 MB + 369 MB
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=4,
                    help="headline shard configuration 1..5 (default 4: the 8B-like 512K zigzag shard, the largest one)")
    ap.add_argument("--head-dim", type=int, default=0,
                    help="variant run: the same shard with this head_dim (64 or 128) instead of the configuration's own")
    ap.add_argument("--only-headline", action="store_true",
                    help="time the headline workload only (no other configurations, no contiguous-chunk replay, no "
                         "HBM-bound kernels, no MFMA probe, no oracle): the command the rocprofv3 summaries are made with")
    ap.add_argument("--no-others", action="store_true", help="skip the other bf16 configurations and the contiguous-chunk replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known HBM traffic) before the timed "
                         "region, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--no-mfma-probe", action="store_true", help="skip the register-only MFMA rate measurement")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows per q segment for the oracle sample (0: auto)")
    return ap.parse_args()


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def measure(w, inputs, steps, warmup, copy_calibration=False):
    """Times `steps` passes of the whole hot path (forward replay, Delta, backward replay) over workload `w` after
    `warmup` untimed ones.  Returns (result dict, ShardRun)."""
    from paper_2605_07569_amd import hexi, replay
    run = replay.ShardRun(w, inputs, "cuda:0", fused_merge=True)
    n_pairs_chunk = [hexi.hexi_shard_mask(w.q_segs, ch, want_pos=False)["n_pairs"] for ch in w.chunks]
    n_pairs = sum(n_pairs_chunk)
    d, nq = w.head_dim, w.n_q_heads
    flops_fwd = 4.0 * d * n_pairs * nq
    flops_bwd = 10.0 * d * n_pairs * nq
    live = [j for j, n in enumerate(n_pairs_chunk) if n > 0]       # chunks that launch the attention kernels
    # the dominant kernel's launches that are timed one by one: the chunks other than the diagonal one(s), i.e.
    # those in which no key lies inside a q segment (all of their tiles are unmasked or invisible)
    def has_diagonal(ch):
        return any(ks < qs + qn and qs < ks + kn for qs, qn in w.q_segs for ks, kn in ch)
    remote = [j for j in live if not has_diagonal(w.chunks[j])]

    for _ in range(warmup):
        run.step()
    torch.cuda.synchronize()
    if copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").fill_(1.0)   # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ev = lambda: torch.cuda.Event(enable_timing=True)
    fwd_ev, bwd_ev, kern_ev = [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        run.forward()
        e1.record()
        # backward replay with events around every bwd_chunk launch (same stream as the kernels)
        run.dq.zero_()
        for j, ch in enumerate(w.chunks):
            flags = hexi.HEXI_COMPUTE_DELTA if j == 0 else 0
            # the step's two kernels are issued through the two halves of the call so that HIP events on the
            # launch stream bracket the dominant one (dK/dV) alone; same launches, same order as one call
            ka, kb = ev(), ev()
            ka.record()
            hexi.hexi_attn_bwd_chunk(run.desc[j], w.q_segs, ch, run.q, run.k[j], run.v[j], run.o, run.d_o,
                                     run.lse, run.delta, None, run.dk[j], run.dv[j], flags=flags | hexi.HEXI_SKIP_DQ)
            kb.record()
            hexi.hexi_attn_bwd_chunk(run.desc[j], w.q_segs, ch, run.q, run.k[j], run.v[j], run.o, run.d_o,
                                     run.lse, run.delta, run.dq, None, None, flags=hexi.HEXI_SKIP_DKDV)
            if j in remote and j != 0:
                kern_ev.append((j, ka, kb))
        e2.record()
        fwd_ev.append((e0, e1))
        bwd_ev.append((e1, e2))
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / steps
    fwd_ms = sum(a.elapsed_time(b) for a, b in fwd_ev) / steps
    bwd_ms = sum(a.elapsed_time(b) for a, b in bwd_ev) / steps
    step_ms = sorted(f[0].elapsed_time(b[1]) for f, b in zip(fwd_ev, bwd_ev))     # per-step device time
    tflops = (flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the dK/dV half of the backward step.  Per launch its algorithmic work is the four
    # matmuls S = QK^T, dP = dO V^T, dV = P^T dO, dK = dS^T Q on the unmasked pairs: 8*d*nq*(pairs of that chunk).
    # (When the launcher splits a GQA group over several workgroups the event pair also covers the two
    # zero-fills of dk/dv that precede the kernel.)
    if kern_ev:
        k_ms = sum(a.elapsed_time(b) for _, a, b in kern_ev) / len(kern_ev)
        k_flops = sum(8.0 * d * nq * n_pairs_chunk[j] for j, _, _ in kern_ev) / len(kern_ev)
    else:  # no remote chunk besides the first: fall back to the whole backward replay
        k_ms, k_flops = bwd_ms, flops_bwd
    achieved = k_flops / (k_ms * 1e-3) / 1e12
    is_bf16 = w.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if is_bf16 else 157.3
    roofline = {"bound": "mfma" if is_bf16 else "alu", "kernel": "bwd_dkdv_bf16_kernel" if is_bf16 else "bwd_f32_kernel",
                "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(w.name), "launch_ms": round(k_ms, 4),
                "flops_per_launch": k_flops, "launches_timed": len(kern_ev) // max(1, steps)}
    res = {"value": round(tflops, 2), "unit": "TFLOP/s", "steps": steps, "warmup": warmup,
           "ms_per_step": round(ms_per_step, 4), "dtype": w.dtype,
           "config": {"workload": w.name, "note": w.note, "n_q_heads": nq, "n_kv_heads": w.n_kv_heads, "head_dim": d,
                      "q_rows": w.lq, "kv_chunks": len(w.chunks), "unmasked_pairs_per_head": n_pairs,
                      "counted_tflop_per_step": round((flops_fwd + flops_bwd) / 1e12, 3)},
           "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
           "step_ms_min": round(step_ms[0], 4), "step_ms_median": round(step_ms[len(step_ms) // 2], 4),
           "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4),
           "fwd_tflops": round(flops_fwd / (fwd_ms * 1e-3) / 1e12, 2),
           "bwd_tflops": round(flops_bwd / (bwd_ms * 1e-3) / 1e12, 2),
           "roofline": roofline}
    # The paper's own cost convention (App. A.4, Eq. 11): 16 * L_q * L_src * n_d * d_h per ring step, no causal
    # discount, recomputation counted as a separate pass; summed here over the steps that see at least one key.
    paper_flops = sum(16.0 * w.lq * sum(n for _, n in w.chunks[j]) * nq * d for j in live)
    res["paper_convention"] = {"tflop_per_step": round(paper_flops / 1e12, 3),
                               "tflops": round(paper_flops / (ms_per_step * 1e-3) / 1e12, 2),
                               "note": "16*Lq*Lc*nq*d per live ring step (App. A.4 Eq. 11), masked pairs included"}
    return res, run, n_pairs


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the ring on one MI355X; --gpus above 1 is not supported "
              "(no collectives are part of this build)", file=sys.stderr)
        sys.exit(2)
    from paper_2605_07569_amd import hexi
    from paper_2605_07569_amd import workloads as wl

    hexi.load()   # raises if the HIP library is not built: no fallback path exists
    torch.cuda.set_device(0)
    w = wl.config(args.workload)
    if args.head_dim and args.head_dim != w.head_dim:
        import dataclasses
        w = dataclasses.replace(w, head_dim=args.head_dim, name=f"{w.name}_d{args.head_dim}",
                                note=w.note + f" (variant: head_dim {args.head_dim})")
    log(f"generating inputs of {w.name} on the host")
    inputs = wl.make_inputs(w)
    log(f"timing {w.name}: {args.warmup} warm-up + {args.steps} steps")
    res, run, n_pairs = measure(w, inputs, args.steps, args.warmup, args.copy_calibration)
    out = {"metric": "attention fwd+bwd TFLOP/s per shard on 1 MI355X; % of bf16 MFMA peak",
           "value": res["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": w.dtype, "data": "synthetic"}
    out.update({k: v for k, v in res.items() if k not in out})
    is_bf16 = w.dtype == "bf16"
    if not args.only_headline:
        out["hbm_bound_kernels"] = hbm_bound_kernels(run, w)
    del run
    torch.cuda.empty_cache()
    if is_bf16 and not args.no_mfma_probe and not args.only_headline:
        out["mfma_probe"] = mfma_probe()
        # context only: frac stays against the nominal peak
        out["roofline"]["frac_of_measured_mfma_rate"] = round(out["roofline"]["achieved"] / out["mfma_probe"]["random_tflops"], 4)

    if not args.only_headline and not args.no_others and not args.head_dim:
        # the zigzag configurations with the alternative reading of "chunk": the same keys as equal contiguous
        # chunks (parity of this chunking is a test; its time stands beside the zigzag-pair replay's)
        contig = {}
        others = {}
        short_steps, short_warm = max(1, min(args.steps, 5)), 2
        for idx in (2, 3, 4, 5):
            wi = wl.config(idx)
            if idx == args.workload:
                inp = inputs
            else:
                log(f"generating inputs of {wi.name}")
                inp = wl.make_inputs(wi)
                log(f"timing {wi.name}: {short_warm} warm-up + {short_steps} steps")
                r, run_i, _ = measure(wi, inp, short_steps, short_warm)
                del run_i
                torch.cuda.empty_cache()
                others[wi.name] = r
            if len(wi.q_segs) == 2:     # a zigzag shard
                wc = wl.contiguous_chunks(wi, len(wi.chunks))
                log(f"timing {wc.name}")
                r, run_i, _ = measure(wc, inp, short_steps, short_warm)
                del run_i
                torch.cuda.empty_cache()
                contig[wc.name] = {k: r[k] for k in ("value", "unit", "ms_per_step", "fwd_tflops", "bwd_tflops", "steps", "warmup")}
            del inp
        out["other_workloads"] = others
        out["contiguous_chunk_replay"] = contig

    if not args.no_cpu_baseline and not args.only_headline:
        log("timing the fp64 oracle on a sample of the headline workload (host cores)")
        out["cpu_baseline"] = cpu_baseline(w, inputs, args.cpu_rows, n_pairs)
    print(json.dumps(out), flush=True)


def mfma_probe(seconds=1.0, iters=100000):
    """What the matrix cores sustain with nothing else going on: a register-only MFMA loop on zero and on
    random bf16 operands, each run for about `seconds` (the clock needs some tenths of a second to settle
    under the load) and timed over its last launches.  Context for `roofline.frac`: the nominal peak assumes 2.4 GHz."""
    from paper_2605_07569_amd import hexi
    dev = torch.device("cuda:0")
    sink = torch.empty(256 * 512, dtype=torch.float32, device=dev)
    flops = 256.0 * 8 * 4 * iters * 32768
    res = {}
    for name, ops in (("zeros", torch.zeros(32768, dtype=torch.bfloat16, device=dev)),
                      ("random", torch.empty(32768, dtype=torch.float32, device=dev).uniform_(-2.5, 2.5).to(torch.bfloat16))):
        t_end = time.perf_counter() + seconds
        ms = []
        while time.perf_counter() < t_end:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            hexi.hexi_mfma_probe(ops, sink, iters)
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        tail = ms[-max(1, len(ms) // 4):]
        res[name + "_tflops"] = round(flops / (sum(tail) / len(tail) * 1e-3) / 1e12, 1)
    res["note"] = "register-only v_mfma_f32_32x32x16_bf16 loop, whole chip; the shader clock is power-limited and depends on the operand bits"
    return res


def hbm_bound_kernels(run, w, reps=10):
    """The HBM-bound steps, outside the timed region: the Delta prepass (reads o fp32 and dO, writes Delta), the
    unfused two-term LSE merge (reads both partials, writes the accumulator) and the head redistribution that
    precedes the all-to-all, each against the 8 TB/s HBM roof with its algorithmic bytes."""
    from paper_2605_07569_amd import hexi
    lq, nq, d = w.lq, w.n_q_heads, w.head_dim
    esz = 2 if w.dtype == "bf16" else 4
    o_part, lse_part = torch.zeros_like(run.o), torch.zeros_like(run.lse)
    o_acc, lse_acc = run.o.clone(), run.lse.clone()

    def timed(fn):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    merge_ms = timed(lambda: hexi.hexi_attn_merge_lse(o_acc, lse_acc, o_part, lse_part))
    merge_bytes = 3.0 * lq * nq * (4 * d + 4)            # read accumulator + partial, write accumulator
    # Delta alone: a backward call with HEXI_COMPUTE_DELTA on a one-key chunk that lies in the shard's future
    # (the call then only fills Delta and zeroes one row of dk/dv)
    last_pos = max(st + n for st, n in w.q_segs)
    k1, v1 = run.k[0][:1].contiguous(), run.v[0][:1].contiguous()
    dk1, dv1 = torch.empty((1, w.n_kv_heads, d), dtype=torch.float32, device=run.dev), torch.empty((1, w.n_kv_heads, d), dtype=torch.float32, device=run.dev)
    desc1 = hexi.desc_for(run.q, k1, w.scale, w.kv_of_q)
    delta_ms = timed(lambda: hexi.hexi_attn_bwd_chunk(desc1, w.q_segs, [(last_pos, 1)], run.q, k1, v1, run.o, run.d_o, run.lse,
                                                      run.delta, run.dq, dk1, dv1, flags=hexi.HEXI_COMPUTE_DELTA))
    delta_bytes = float(lq) * nq * (d * (4 + esz) + 4)   # read o (fp32) and dO, write Delta
    # head redistribution before the all-to-all (Sec. 3.2): the shard's fused Q|K|V tensor cut into the parts of
    # three ranks with uneven head counts (half, a third and a sixth of the q heads, plus the kv heads they need)
    nkv = w.n_kv_heads
    fused = torch.empty((lq, nq + 2 * nkv, d), dtype=run.q.dtype, device=run.dev).normal_()
    cuts = [0, nq // 2, nq // 2 + nq // 3, nq]
    lists = []
    for r in range(3):
        heads = list(range(cuts[r], cuts[r + 1]))
        kv = sorted({w.kv_of_q[h] if w.kv_of_q else h // (nq // nkv) for h in heads})
        lists.append(heads + [nq + k for k in kv] + [nq + nkv + k for k in kv])
    listed = sum(len(l) for l in lists)
    packed = torch.empty((listed * lq * d,), dtype=run.q.dtype, device=run.dev)
    pack_ms = timed(lambda: hexi.hexi_a2a_pack(fused, packed, lists))
    a2a_bytes = 2.0 * listed * lq * d * esz              # every listed element read once and written once
    res = {"a2a_pack": {"ms": round(pack_ms, 4), "GB/s": round(a2a_bytes / pack_ms / 1e6, 1),
                        "frac_of_8TBps": round(a2a_bytes / pack_ms / 1e6 / 8000.0, 3), "MB_moved": round(a2a_bytes / 1e6, 1)}}
    res.update({"merge_lse": {"ms": round(merge_ms, 4), "GB/s": round(merge_bytes / merge_ms / 1e6, 1),
                         "frac_of_8TBps": round(merge_bytes / merge_ms / 1e6 / 8000.0, 3)}})
    if delta_ms > 0:
        res["delta"] = {"ms": round(delta_ms, 4), "GB/s": round(delta_bytes / delta_ms / 1e6, 1),
                        "frac_of_8TBps": round(delta_bytes / delta_ms / 1e6 / 8000.0, 3)}
    return res


def cpu_baseline(w, inputs, rows_per_seg, n_pairs_full=None):
    """The fp64 oracle, as it stands, on a bounded sample: a few rows of every q segment, all local
    heads, each row against all its visible keys, forward + backward.  Rate in the metric's unit,
    counting the same 14*d flops per unmasked pair."""
    import numpy as np
    import oracle
    from paper_2605_07569_amd import workloads as wl
    q_pos_all = wl.seg_positions(w.q_segs).numpy()
    if rows_per_seg <= 0:
        # aim at ~1e8 (row, key, head) triples: 10-30 s of oracle work on 16 cores
        budget = 1.0e8
        per_row = float(np.mean(q_pos_all + 1)) * w.n_q_heads
        rows_per_seg = max(1, int(budget / per_row / len(w.q_segs)))
    rows, off = [], 0
    for s, n in w.q_segs:
        take = min(rows_per_seg, n)
        rows.extend(off + np.linspace(0, n - 1, take).astype(np.int64))
        off += n
    rows = np.array(sorted(set(int(r) for r in rows)), dtype=np.int64)
    q_pos = q_pos_all[rows]
    n_keys = int(q_pos.max()) + 1
    f64 = lambda t: t.to(torch.float64).numpy()
    q, d_o = f64(inputs["q"][rows]), f64(inputs["d_o"][rows])
    k, v = f64(inputs["k"][:n_keys]), f64(inputs["v"][:n_keys])
    kv_pos = np.arange(n_keys, dtype=np.int64)
    t0 = time.perf_counter()
    oracle.attn_fwd(q, q_pos, k, v, kv_pos, w.scale, w.kv_of_q)
    oracle.attn_bwd(q, q_pos, k, v, kv_pos, d_o, w.scale, w.kv_of_q)
    dt = time.perf_counter() - t0
    pairs = float(np.sum(q_pos + 1))
    flops = 14.0 * w.head_dim * pairs * w.n_q_heads
    extra = {}
    if n_pairs_full:
        extra["extrapolated_full_seconds"] = round(dt * n_pairs_full / pairs, 0)    # an extrapolation, not a measurement
    return {**extra, "value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{len(rows)} of {w.lq} shard rows (evenly spaced in each q segment) x all {w.n_q_heads} local heads, "
                      f"each against all its visible keys, fwd+bwd in fp64; {dt:.1f} s",
            "seconds": round(dt, 2)}


if __name__ == "__main__":
    main()
