#!/usr/bin/env python3
"""Benchmark of the PrefixKV hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: prefixkv_importance -> prefixkv_select -> prefixkv_compact -> T decode steps of
prefixkv_decode_attn (append + attention over all layers).  The headline value is the compressed
decode throughput B*T / (time of the decode loop); prefixkv_select ms and the other stages are
reported beside it.  Prints ONE JSON line.

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
    Bk = w.budget_tokens(r)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    K, W, T = args.steps, args.warmup, w.decode_steps

    x = make_prefill(w, device=dev)
    dec = make_decode(w, device=dev)
    hp = HotPath(x["q"], x["k"], x["v"], x["scale"], Bk, T, evict_distance=args.evict_distance)
    dq, dk, dv = dec["q"], dec["k"], dec["v"]
    use_graph = not args.no_graph

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

    stage_ms = [sum(evs[i][j].elapsed_time(evs[i][j + 1]) for i in range(K)) / K for j in range(4)]
    imp_ms, sel_ms, cmp_ms, dec_ms = stage_ms
    tok_s = w.B * T / (dec_ms * 1e-3)
    d_ev = args.evict_distance
    if d_ev is None:
        assert int(hp.cache.lens.sum()) == int(lens0.sum()) + w.B * w.L * T, "decode loop did not run to the end"
        step_tokens = [None] * T
    else:
        assert int(hp.cache.lens.sum()) + w.B * w.L * min(T, d_ev) == cached_tokens_under_pruning(lens0, w.N, T, d_ev), \
            "decode loop did not run to the end"
        step_tokens = [cached_tokens_under_pruning(lens0, w.N, t + 1, d_ev) for t in range(T)]

    # ---- roofline of the dominant kernel (decode_attn_kernel).  The decode loop is T launches of that
    # one kernel and nothing else, back to back on one stream (a HIP graph by default), so the event
    # time of the loop divided by T is the kernel's average launch duration over the timed region.
    n_seg, esz = w.B * w.L, w.elem_bytes
    kern_ms = dec_ms / T
    lens0_sum = int(lens0.sum())
    alg_bytes = sum(algorithmic_decode_bytes(lens0_sum, n_seg, t, w.H, w.Hkv, w.D, esz, step_tokens[t])
                    for t in range(T)) / T
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        key = f"decode_attn_kernel/{w.name}/budget{r:g}" + ("" if d_ev is None else f"/evict{d_ev}")
        traffic = json.load(open(tpath)).get(key)
    gqa = w.dtype == "bf16" and (w.H // w.Hkv) % 2 == 0
    roofline = {"kernel": "decode_plan_kernel + decode_gqa_kernel" if gqa else "decode_attn_kernel", "bound": "hbm", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "bytes_per_launch": int(alg_bytes), "kernel_ms": round(kern_ms, 5),
                "launches_per_step": T,
                "first_launch_bytes": algorithmic_decode_bytes(lens0_sum, n_seg, 0, w.H, w.Hkv, w.D, esz,
                                                               step_tokens[0]),
                "last_launch_bytes": algorithmic_decode_bytes(lens0_sum, n_seg, T - 1, w.H, w.Hkv, w.D, esz,
                                                              step_tokens[T - 1])}
    flops = 2 * w.B * w.L * w.H * w.N * (w.N + 1) * w.D   # two causal QK^T passes (lse, column sums)
    imp_tflops = flops / (imp_ms * 1e-3) / 1e12
    cmp_bytes = 2 * lens0_sum * w.Hkv * w.D * esz * 2 + w.B * w.L * w.N * 4
    extra = {
        "importance": {"ms": round(imp_ms, 4), "tflops": round(imp_tflops, 1),
                       "frac_mfma_bf16": round(imp_tflops / MFMA_BF16_PEAK_TFLOPS, 4), "passes": 2},
        "select": {"ms": round(sel_ms, 4), "iters": hp.sel.iters.tolist()[:4], "p": hp.sel.p.tolist()[:2]},
        "compact": {"ms": round(cmp_ms, 4), "GBps": round(cmp_bytes / (cmp_ms * 1e-3) / 1e9, 1)},
        "decode_loop": {"ms": round(dec_ms, 4), "us_per_decode_step": round(dec_ms * 1e3 / T, 2),
                        "graph": use_graph},
    }

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, x, dec, hp, Bk)
    extras = time_extras(P, w, x, hp, Bk, T) if args.extras else None

    line = {
        "metric": "compressed decode tok/s (attention over all layers per step) + prefixkv_select ms; "
                  "LLaVA-7B shape, 20% budget",
        "value": round(tok_s, 1), "unit": "tok/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(wall * 1e3 / K, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "L": w.L, "H": w.H, "Hkv": w.Hkv, "D": w.D, "N": w.N,
                   "budget": r, "budget_tokens": Bk, "decode_steps": T,
                   "decode_mode": "append" if d_ev is None else f"prune at distance {d_ev}"},
        "prefixkv_select_ms": round(sel_ms, 4),
        "stages": extra, "roofline": roofline, "cpu_baseline": cpu,
    }
    if extras is not None:
        line["extras"] = extras
    print(json.dumps(line))
    return 0


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
        out["importance_with_lse"] = {"ms": round(t, 4), "tflops": round(flops1 / t / 1e9, 1), "passes": 1}
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
    workload: stages 2+3 in full, and the first decode steps of sequence 0."""
    import numpy as np
    import oracle
    f = lambda t: t.detach().float().cpu().numpy()
    cores = oracle.threads()
    imp = hp.importance[:1].cpu().numpy()
    t0 = time.perf_counter()
    sel = oracle.select(imp, Bk)
    sel_s = time.perf_counter() - t0
    n_dec = min(w.decode_steps, 32)
    cache = oracle.compact(f(x["k"][:1]), f(x["v"][:1]), sel["order"], sel["lengths"], n_dec)
    scale = x["scale"].cpu().numpy()
    dq, dk, dv = f(dec["q"][:n_dec, :1]), f(dec["k"][:n_dec, :1]), f(dec["v"][:n_dec, :1])
    t0 = time.perf_counter()
    for t in range(n_dec):
        oracle.decode_attn(cache, dq[t], dk[t], dv[t], scale, out_bf16=(w.dtype == "bf16"))
    dec_s = time.perf_counter() - t0
    return {"value": round(n_dec / dec_s, 2), "unit": "tok/s", "cores": cores, "kind": "oracle",
            "sample": f"sequence 0 of {w.B}: first {n_dec} of {w.decode_steps} decode steps, all {w.L} layers "
                      f"(fp64 oracle, OpenMP); select of 1 sequence took {sel_s * 1e3:.1f} ms",
            "select_ms_per_sequence": round(sel_s * 1e3, 2)}


if __name__ == "__main__":
    sys.exit(main())
