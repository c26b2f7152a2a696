#!/usr/bin/env python3
"""Benchmark of the PrefixKV hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: prefixkv_importance -> prefixkv_select -> prefixkv_compact -> T decode steps of
prefixkv_decode_attn (append + attention over all layers).  The headline value is the compressed
decode throughput B*T / (time of the decode loop); prefixkv_select ms and the other stages are
reported beside it (medians over the timed steps), together with the same decode loop over the
uncompressed cache ("full_cache"), the batch-16 companion of the default workload ("companion") and the
CPU oracle timed on a bounded sample ("cpu_baseline").  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config llava7b_b1] [--budget r]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def algorithmic_decode_bytes(lens0_sum: int, n_seg: int, t: int, H: int, Hkv: int, D: int, esz: int,
                             tokens: int = None) -> int:
    """HBM bytes the method itself must move in decode step t (0-based): every occupied slot of K and V
    once (including the token appended in this step), q in, out out, and the appended k/v written."""
    if tokens is None:
        tokens = lens0_sum + n_seg * (t + 1)
    return tokens * Hkv * D * esz * 2 + n_seg * (2 * H + 2 * Hkv) * D * esz


def cached_tokens_under_pruning(lens0, N: int, t: int, d: int) -> int:
    """Entries cached after 1-based step t when decoding with pruning at distance d, summed over all
    segments: max(target(t), k + min(t, d)) with target = round-half-up(k (N+t) / N), at least 1."""
    k = lens0.to("cpu").long()
    target = ((2 * k * (N + t) + N) // (2 * N)).clamp(min=1)
    return int(torch.maximum(target, k + min(t, d)).sum())


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="llava7b_b1")
    ap.add_argument("--budget", type=float, default=None)
    ap.add_argument("--decode-steps", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None, help="override the batch size of the workload")
    ap.add_argument("--evict-distance", type=int, default=None, metavar="D",
                    help="decode with pruning at distance D from the newest token instead of append-only")
    ap.add_argument("--no-graph", action="store_true", help="launch every decode step from Python")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-cache", action="store_true",
                    help="skip the decode loop over the uncompressed cache (the speed-up comparator)")
    ap.add_argument("--no-companion", action="store_true",
                    help="skip the batch-16 companion measurement of the default workload")
    ap.add_argument("--extras", action="store_true",
                    help="also time the entry points beyond the core path (prefill attention, one-pass importance, "
                         "ranking + offline configuration, Gini, positional and feature merging) and add them to "
                         "the line as \"extras\"")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="BYTES",
                    help="only run the plain copy kernel on BYTES (for calibrating rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU (the path shards over the batch with no exchange); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2

    import paper_2412_03409_amd as P
    from paper_2412_03409_amd.pipeline import HotPath
    from pkv_workloads import CONFIGS, make_decode, make_prefill

    P.load()
    if args.calibrate_copy:
        n = args.calibrate_copy // 16 * 16
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
        for _ in range(5):
            P.prefixkv_calibration_copy(dst, src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration_copy_bytes": n, "launches": 5}))
        return 0
    w = CONFIGS[args.config]
    if args.decode_steps is not None:
        w = w.with_(decode_steps=args.decode_steps)
    if args.batch is not None:
        w = w.with_(B=args.batch)
    r = w.budget if args.budget is None else args.budget
    torch.cuda.set_device(0)
    K, W = args.steps, args.warmup
    use_graph = not args.no_graph

    m = measure(P, HotPath, w, r, K, W, use_graph, args.evict_distance)
    hp, x, dec, Bk, T = m.pop("hp"), m.pop("x"), m.pop("dec"), m["budget_tokens"], w.decode_steps

    # ---- the same decode loop over the uncompressed cache (every layer keeps all N positions): what the
    # compression buys on this chip.  Attention only, like the headline value.
    full = None
    if not args.no_full_cache and args.evict_distance is None:
        full = decode_only(P, HotPath, w, 1.0, max(3, min(K, 5)), use_graph, x=x, dec=dec)
        full = {"tok_s": full["tok_s"], "us_per_decode_step": full["us_per_decode_step"],
                "GBps": full["roofline"]["achieved"], "frac_hbm": full["roofline"]["frac"],
                "bytes_per_launch": full["roofline"]["bytes_per_launch"]}
        full["speedup_of_compressed"] = round(m["tok_s"] / full["tok_s"], 3)

    cpu = None if args.no_cpu_baseline else cpu_baseline(w, x, dec, hp, Bk)
    extras = time_extras(P, w, x, hp, Bk, T) if args.extras else None
    del hp, x, dec
    torch.cuda.empty_cache()

    # ---- companion: the batch-16 workload at the same budget.  The batch-1 working set (73-207 MB) sits in
    # the chip's 256 MB last-level cache; this one (1.1-2.2 GB per step) cannot, so its fraction of the HBM
    # peak is the bandwidth-honest one.
    companion = None
    if not args.no_companion and args.config == "llava7b_b1" and args.evict_distance is None and args.batch is None:
        wc = CONFIGS["llava7b_b16"]
        c = decode_only(P, HotPath, wc, r, 3, use_graph, stages=True)
        companion = {"workload": wc.name, "B": wc.B, "budget": r, "decode_steps": wc.decode_steps, "timed_loops": 3,
                     "tok_s": c["tok_s"], "us_per_decode_step": c["us_per_decode_step"], "roofline": c["roofline"],
                     "stages": c["stages"]}

    line = {
        "metric": "compressed decode tok/s (attention over all layers per step) + prefixkv_select ms; "
                  "LLaVA-7B shape, 20% budget",
        "value": m["tok_s"], "unit": "tok/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "L": w.L, "H": w.H, "Hkv": w.Hkv, "D": w.D, "N": w.N,
                   "budget": r, "budget_tokens": Bk, "decode_steps": T,
                   "decode_mode": "append" if args.evict_distance is None else f"prune at distance {args.evict_distance}"},
        "prefixkv_select_ms": m["stages"]["select"]["ms"],
        "stages": m["stages"], "roofline": m["roofline"], "cpu_baseline": cpu,
        "full_cache": full, "speedup_vs_full_cache": None if full is None else full["speedup_of_compressed"],
        "companion": companion, "timing": "median of the timed steps (HIP events on the launch stream)",
    }
    if extras is not None:
        line["extras"] = extras
    print(json.dumps(line))
    return 0


def _median(v):
    v = sorted(v)
    n = len(v)
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def _decode_source_digest():
    import hashlib
    h = hashlib.sha256()
    for f in ("decode.hip", "pkv_common.hpp"):
        with open(os.path.join(ROOT, "paper_2412_03409_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def decode_roofline(w, r, lens0, T, dec_ms, d_ev=None):
    """Roofline of the decode launch.  The decode loop is T launches of one kernel (for grouped-query bf16
    caches: a planning kernel and the attention kernel, timed together) and nothing else, back to back on one
    stream (a HIP graph by default), so the event time of the loop divided by T is the average launch
    duration over the timed region."""
    n_seg, esz = w.B * w.L, w.elem_bytes
    lens0_sum = int(lens0.sum())
    if d_ev is None:
        step_tokens = [None] * T
    else:
        step_tokens = [cached_tokens_under_pruning(lens0, w.N, t + 1, d_ev) for t in range(T)]
    kern_ms = dec_ms / T
    alg_bytes = sum(algorithmic_decode_bytes(lens0_sum, n_seg, t, w.H, w.Hkv, w.D, esz, step_tokens[t])
                    for t in range(T)) / T
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        # counter values belong to the kernel source they were measured on: a changed source reports null
        # until the PMC passes have been run again
        table = json.load(open(tpath))
        if table.get("_decode_source_sha256") == _decode_source_digest():
            key = f"decode_attn_kernel/{w.name}/budget{r:g}" + ("" if d_ev is None else f"/evict{d_ev}")
            traffic = table.get(key)
    gqa = w.dtype == "bf16" and (w.H // w.Hkv) % 2 == 0
    return {"kernel": "decode_plan_kernel + decode_gqa_kernel" if gqa else "decode_attn_kernel", "bound": "hbm",
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "bytes_per_launch": int(alg_bytes),
            "kernel_ms": round(kern_ms, 5), "launches_per_step": T,
            "first_launch_bytes": algorithmic_decode_bytes(lens0_sum, n_seg, 0, w.H, w.Hkv, w.D, esz, step_tokens[0]),
            "last_launch_bytes": algorithmic_decode_bytes(lens0_sum, n_seg, T - 1, w.H, w.Hkv, w.D, esz,
                                                          step_tokens[T - 1])}


def measure(P, HotPath, w, r, K, W, use_graph, d_ev=None, x=None, dec=None):
    """W untimed and K timed passes of the whole hot path on resident inputs; stage times are medians."""
    from pkv_workloads import make_decode, make_prefill
    dev = "cuda:0"
    Bk, T = w.budget_tokens(r), w.decode_steps
    x = make_prefill(w, device=dev) if x is None else x
    dec = make_decode(w, device=dev) if dec is None else dec
    hp = HotPath(x["q"], x["k"], x["v"], x["scale"], Bk, T, evict_distance=d_ev)
    dq, dk, dv = dec["q"], dec["k"], dec["v"]

    # first pass also validates the run (status words, budget met)
    hp.run_importance(); hp.run_select(); hp.run_compact()
    torch.cuda.synchronize()
    assert int(hp.sel.status.abs().sum()) == 0, "select reported a data error"
    lens0 = hp.sel.lengths.clone()
    assert (lens0.sum(dim=1) == min(Bk, w.L * w.N)).all(), "budget not met"
    if use_graph:
        hp.capture_decode_loop(dq, dk, dv)

    def one_step(ev=None):
        if ev: ev[0].record()
        hp.run_importance()
        if ev: ev[1].record()
        hp.run_select()
        if ev: ev[2].record()
        hp.run_compact()
        if ev: ev[3].record()
        if use_graph:
            hp.replay_decode_loop()
        else:
            hp.run_decode_loop(dq, dk, dv)
        if ev: ev[4].record()

    for _ in range(W):
        one_step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
    t0 = time.perf_counter()
    for i in range(K):
        one_step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    imp_ms, sel_ms, cmp_ms, dec_ms = [_median([evs[i][j].elapsed_time(evs[i][j + 1]) for i in range(K)])
                                      for j in range(4)]
    tok_s = w.B * T / (dec_ms * 1e-3)
    if d_ev is None:
        assert int(hp.cache.lens.sum()) == int(lens0.sum()) + w.B * w.L * T, "decode loop did not run to the end"
    else:
        assert int(hp.cache.lens.sum()) + w.B * w.L * min(T, d_ev) == cached_tokens_under_pruning(lens0, w.N, T, d_ev), \
            "decode loop did not run to the end"
    esz = w.elem_bytes
    # two causal QK^T products per head (the row lse, then the column sums), both inside one kernel that
    # reads Q and K from HBM once
    flops = 2 * w.B * w.L * w.H * w.N * (w.N + 1) * w.D
    imp_tflops = flops / (imp_ms * 1e-3) / 1e12
    cmp_bytes = 2 * int(lens0.sum()) * w.Hkv * w.D * esz * 2 + w.B * w.L * w.N * 4
    stages = {
        "importance": {"ms": round(imp_ms, 4), "tflops": round(imp_tflops, 1),
                       "frac_mfma_bf16": round(imp_tflops / MFMA_BF16_PEAK_TFLOPS, 4), "products": 2, "kernels": 1},
        "select": {"ms": round(sel_ms, 4), "iters": hp.sel.iters.tolist()[:4], "p": hp.sel.p.tolist()[:2]},
        "compact": {"ms": round(cmp_ms, 4), "GBps": round(cmp_bytes / (cmp_ms * 1e-3) / 1e9, 1)},
        "decode_loop": {"ms": round(dec_ms, 4), "us_per_decode_step": round(dec_ms * 1e3 / T, 2),
                        "graph": use_graph},
    }
    return {"tok_s": round(tok_s, 1), "ms_per_step": round(wall * 1e3 / K, 4), "stages": stages,
            "roofline": decode_roofline(w, r, lens0, T, dec_ms, d_ev), "budget_tokens": Bk,
            "us_per_decode_step": round(dec_ms * 1e3 / T, 2), "hp": hp, "x": x, "dec": dec}


def decode_only(P, HotPath, w, r, K, use_graph, x=None, dec=None, stages=False):
    """Builds the cache of workload w at budget r once, then times K runs of its decode loop (one warm-up);
    with stages=True importance / select / compact are timed as well (median of K)."""
    from pkv_workloads import make_decode, make_prefill
    dev = "cuda:0"
    Bk, T = w.budget_tokens(r), w.decode_steps
    x = make_prefill(w, device=dev) if x is None else x
    dec = make_decode(w, device=dev) if dec is None else dec
    hp = HotPath(x["q"], x["k"], x["v"], x["scale"], Bk, T)
    hp.run_importance(); hp.run_select(); hp.run_compact()
    torch.cuda.synchronize()
    assert int(hp.sel.status.abs().sum()) == 0, "select reported a data error"
    lens0 = hp.sel.lengths.clone()
    assert (lens0.sum(dim=1) == min(Bk, w.L * w.N)).all(), "budget not met"
    dq, dk, dv = dec["q"], dec["k"], dec["v"]
    if use_graph:
        hp.capture_decode_loop(dq, dk, dv)
    times = [[] for _ in range(4)]
    for i in range(K + 1):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        ev[0].record()
        if stages: hp.run_importance()
        ev[1].record()
        if stages: hp.run_select()
        ev[2].record()
        hp.run_compact()
        ev[3].record()
        if use_graph:
            hp.replay_decode_loop()
        else:
            hp.run_decode_loop(dq, dk, dv)
        ev[4].record()
        torch.cuda.synchronize()
        if i > 0:
            for j in range(4):
                times[j].append(ev[j].elapsed_time(ev[j + 1]))
    assert int(hp.cache.lens.sum()) == int(lens0.sum()) + w.B * w.L * T, "decode loop did not run to the end"
    imp_ms, sel_ms, cmp_ms, dec_ms = [_median(t) for t in times]
    out = {"tok_s": round(w.B * T / (dec_ms * 1e-3), 1), "us_per_decode_step": round(dec_ms * 1e3 / T, 2),
           "roofline": decode_roofline(w, r, lens0, T, dec_ms)}
    if stages:
        flops = 2 * w.B * w.L * w.H * w.N * (w.N + 1) * w.D
        cmp_bytes = 2 * int(lens0.sum()) * w.Hkv * w.D * w.elem_bytes * 2 + w.B * w.L * w.N * 4
        out["stages"] = {"importance_ms": round(imp_ms, 4),
                         "importance_frac_mfma_bf16": round(flops / (imp_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                         "select_ms": round(sel_ms, 4), "compact_ms": round(cmp_ms, 4),
                         "compact_GBps": round(cmp_bytes / (cmp_ms * 1e-3) / 1e9, 1)}
    del hp
    return out


def time_extras(P, w, x, hp, Bk, T, reps=5):
    """Average time (ms, HIP events on the current stream) of the entry points beyond the core path, on the
    same resident inputs.  The two merges rewrite the compacted cache, so they come last."""
    import torch
    dev = x["q"].device

    def ms(fn, n=reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    out = {}
    flops1 = w.B * w.L * w.H * w.N * (w.N + 1) * w.D           # one causal product
    if w.dtype == "bf16":
        o = torch.empty_like(x["q"])
        lse = torch.empty((w.B, w.L, w.H, w.N), dtype=torch.float32, device=dev)
        t = ms(lambda: P.prefixkv_prefill_attn(x["q"], x["k"], x["v"], x["scale"], out=o, lse=lse))
        out["prefill_attn"] = {"ms": round(t, 4), "tflops": round(2 * flops1 / t / 1e9, 1)}
        t = ms(lambda: P.prefixkv_importance(x["q"], x["k"], x["scale"], lse=lse))
        out["importance_with_lse"] = {"ms": round(t, 4), "tflops": round(flops1 / t / 1e9, 1), "products": 1, "kernels": 1}
        del o
    rk = P.prefixkv_rank(hp.importance)
    out["rank"] = {"ms": round(ms(lambda: P.prefixkv_rank(hp.importance, out=rk)), 4)}
    samples = hp.sel.lengths[:1].repeat(10, 1).contiguous()      # ten calibration samples of this shape
    cfg = P.prefixkv_offline_config(samples, w.N, Bk, w.B)
    out["offline_config"] = {"ms": round(ms(lambda: P.prefixkv_offline_config(samples, w.N, Bk, w.B, out=cfg)), 4),
                             "samples": 10}
    g = P.prefixkv_gini(hp.sel.cum)
    out["gini"] = {"ms": round(ms(lambda: P.prefixkv_gini(hp.sel.cum, out=g)), 4),
                   "min": round(float(g.min()), 4), "max": round(float(g.max()), 4)}
    hp.run_compact()
    rows = 2 * w.B * w.L * w.Hkv * w.N * w.D * w.elem_bytes      # every row of K and V is read once
    t = ms(lambda: P.prefixkv_merge_position(hp.cache, x["k"], x["v"]))
    out["merge_position"] = {"ms": round(t, 4), "GBps_rows_read": round(rows / t / 1e6, 1)}
    if w.dtype == "bf16":
        hp.run_compact()
        match = torch.empty((2, w.B, w.L, w.Hkv, w.N), dtype=torch.int32, device=dev)
        need = P.prefixkv_workspace_bytes(P.binding.OP_MERGE_FEATURE, w.B, w.L, w.H, w.Hkv, w.N, w.D, P.PKV_BF16)
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        t = ms(lambda: P.prefixkv_merge_feature(hp.cache, x["k"], x["v"], match=match, ws=ws), 3)
        mflops = 2.0 * 2 * w.Hkv * w.D * w.N * float(hp.sel.lengths.sum())
        out["merge_feature"] = {"ms": round(t, 4), "matching_tflops_overall": round(mflops / t / 1e9, 1)}
    return out


def cpu_baseline(w, x, dec, hp, Bk):
    """The CPU oracle as it stands, timed on this machine's host cores on a bounded sample of the same
    workload (about 10-30 s of CPU work): every stage for sequence 0 -- importance in full for prompts up to
    1024 positions, else one (sequence, layer) slice with the extrapolation stated --, stages 2+3, compaction,
    and the first decode steps."""
    import numpy as np
    import oracle
    f = lambda t: t.detach().float().cpu().numpy()
    cores = oracle.threads()
    scale = x["scale"].cpu().numpy()
    # stage 1
    n_l = w.L if w.N <= 1024 else 1
    q0, k0 = f(x["q"][:1, :n_l]), f(x["k"][:1, :n_l])
    t0 = time.perf_counter()
    oracle.importance(q0, k0, scale[:n_l])
    imp_s = time.perf_counter() - t0
    imp_seq_ms = imp_s * 1e3 * (w.L / n_l)
    del q0, k0
    # stages 2+3 on the importance the GPU produced
    imp = hp.importance[:1].cpu().numpy()
    t0 = time.perf_counter()
    sel = oracle.select(imp, Bk)
    sel_s = time.perf_counter() - t0
    # stage 4a
    n_dec = min(w.decode_steps, 32)
    k1, v1 = f(x["k"][:1]), f(x["v"][:1])
    t0 = time.perf_counter()
    cache = oracle.compact(k1, v1, sel["order"], sel["lengths"], n_dec)
    cmp_s = time.perf_counter() - t0
    del k1, v1
    # stage 4b
    dq, dk, dv = f(dec["q"][:n_dec, :1]), f(dec["k"][:n_dec, :1]), f(dec["v"][:n_dec, :1])
    t0 = time.perf_counter()
    for t in range(n_dec):
        oracle.decode_attn(cache, dq[t], dk[t], dv[t], scale, out_bf16=(w.dtype == "bf16"))
    dec_s = time.perf_counter() - t0
    imp_note = (f"importance of all {w.L} layers" if n_l == w.L else
                f"importance of layer 0 only ({imp_s:.1f} s), times {w.L} layers as an extrapolation")
    return {"value": round(n_dec / dec_s, 2), "unit": "tok/s", "cores": cores, "kind": "oracle",
            "sample": f"sequence 0 of {w.B} (fp64 oracle, OpenMP): {imp_note}; select and compaction in full; "
                      f"first {n_dec} of {w.decode_steps} decode steps over all {w.L} layers (the tok/s value)",
            "importance_ms_per_sequence": round(imp_seq_ms, 1),
            "importance_extrapolated": n_l != w.L,
            "select_ms_per_sequence": round(sel_s * 1e3, 2),
            "compact_ms_per_sequence": round(cmp_s * 1e3, 2)}


if __name__ == "__main__":
    sys.exit(main())
