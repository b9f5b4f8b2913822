#!/usr/bin/env python3
"""Benchmark of the sparse-incidence KGE training step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic triplets that already sit in
HBM: negative sampling, incidence build (A and sorted A^T), forward (gather product + distance +
margin-ranking loss), backward (transposed product) and the sparse SGD update.  Steps walk the
workload's batches in stored order, epoch after epoch (the last batch of an epoch is partial).

Prints ONE JSON line; see DESIGN.md for the byte model behind "roofline".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="mid", help="workload name: tiny | mid | toruse (and later transh, transr)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=0, help="oracle steps to time (0 = pick for ~10-20 s)")
    return ap.parse_args()


def algorithmic_bytes(wl, rows, touched):
    """Bytes the method itself moves per call for a stacked (TransE/TorusE) step:
    forward  = rows * (3 gathered table rows + 12 B of column ids + 1 dL/dx row written + 4 B score)
    backward = rows * (3 dL/dx rows read, one per entry of A^T, + 3 * 4 B packed entries) + touched * (row + 8 B)
    sgd      = touched * (table row read + gradient row read + table row written)"""
    row = 4 * wl.dim
    fwd = rows * (3 * row + 12 + row + 4)
    bwd = rows * (3 * row + 12) + touched * (row + 8)
    sgd = touched * 3 * row
    return fwd, bwd, sgd


def cpu_baseline(wl, h, r, t, tabs, n_steps):
    """The CPU oracle as it stands, single thread, on the first batches of the same workload."""
    from oracle import stxo
    from tests.util import oracle_batch, oracle_config, oracle_tables
    cfg = oracle_config(wl)
    tb = oracle_tables(tabs)
    slices = [(s, min(s + wl.batch, wl.n_triplets)) for s in range(0, wl.n_triplets, wl.batch)]
    rows = 0
    t0 = time.perf_counter()
    done = 0
    for i in range(n_steps):
        lo, hi = slices[i % len(slices)]
        bt = oracle_batch(wl, h, r, t, lo, hi)
        stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
        stxo.train_step(cfg, tb, bt, wl.lr)
        rows += bt.rows
        done += 1
    dt = time.perf_counter() - t0
    return rows / dt, done, dt


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); rerun with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2502_16949_amd import binding as B
    from paper_2502_16949_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    wl = W.WORKLOADS[args.config]
    if wl.model not in ("transe", "toruse"):
        print(f"bench.py: workload {wl.name} is not benchmarked yet", file=sys.stderr)
        sys.exit(2)

    h, r, t = W.make_graph(wl)
    tabs = W.make_tables(wl)
    hd, rd, td = (torch.from_numpy(a).to(dev) for a in (h, r, t))
    cfg = B.make_config(wl.model, wl.dist, wl.n_ent, wl.n_rel, wl.dim, wl.batch, wl.n_neg, margin=wl.margin)
    ctx = B.Context(cfg, dev)
    params = B.Params(torch.from_numpy(tabs["ent"]).to(dev))
    inc = B.Incidence(ctx)
    grads = B.Grads(ctx)
    scores = torch.empty(ctx.rows_max, dtype=torch.float32, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    nh = torch.empty(wl.batch * wl.n_neg, dtype=torch.int32, device=dev)
    nt = torch.empty(wl.batch * wl.n_neg, dtype=torch.int32, device=dev)
    slices = W.batch_slices(wl)
    seed = W.negative_seed(wl)

    def step(i, ev=None):
        lo, hi = slices[i % len(slices)]
        hb, rb, tb = hd[lo:hi], rd[lo:hi], td[lo:hi]
        if ev: ev[0].record()
        B.stx_sample_negatives(ctx, hb, rb, tb, wl.n_neg, seed, 0, wl.n_triplets, lo, nh, nt)
        if ev: ev[1].record()
        B.stx_build_incidence(ctx, hb, rb, tb, nh, nt, wl.n_neg, inc)
        if ev: ev[2].record()
        B.stx_forward(ctx, inc, params, scores, loss)
        if ev: ev[3].record()
        B.stx_backward(ctx, inc, params, grads)
        if ev: ev[4].record()
        B.stx_sgd_step(ctx, params, inc, grads, wl.lr)
        if ev: ev[5].record()
        return (hi - lo) * (1 + wl.n_neg)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly --steps steps, events on the stream the kernels run on --------------
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    rows_done = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        rows_done += step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    phase = np.zeros(5)
    fwd_full = []
    for i, ev in enumerate(events):
        for p in range(5):
            phase[p] += ev[p].elapsed_time(ev[p + 1])
        lo, hi = slices[(args.warmup + i) % len(slices)]
        if hi - lo == wl.batch:
            fwd_full.append(ev[2].elapsed_time(ev[3]))
    phase_us = phase / args.steps * 1e3
    loss_last = float(loss.item())
    u_last = int(inc.n_touched.item())

    # ---- roofline of the dominant kernel: the fused forward, one launch per full batch --------------
    fwd_bytes, bwd_bytes, sgd_bytes = algorithmic_bytes(wl, wl.rows_per_batch, u_last)
    fwd_ms = float(np.mean(fwd_full)) if fwd_full else float("nan")
    achieved = fwd_bytes / (fwd_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "k_forward_stacked", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "bytes_per_launch": fwd_bytes, "avg_launch_us": round(fwd_ms * 1e3, 2)}

    out = {
        "metric": "training triplets/sec (pos+neg) TransE d=128 fp32" if wl.name == "mid"
                  else f"training triplets/sec (pos+neg) {wl.model} d={wl.dim} fp32",
        "value": round(rows_done / dt, 1), "unit": "triplets/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.model} {wl.dist}, {wl.n_ent} entities, {wl.n_rel} relations, "
                               f"{wl.n_triplets} triplets (Zipf {wl.zipf_ent}/{wl.zipf_rel}), dim {wl.dim}, "
                               f"batch {wl.batch}, {wl.n_neg} negative(s) per positive, margin {wl.margin}, "
                               f"SGD lr {wl.lr}",
                   "rows_per_full_batch": wl.rows_per_batch, "batches_per_epoch": len(slices),
                   "step": "sample negatives + build incidence + forward + backward + sgd"},
        "phase_us": {k: round(float(v), 2) for k, v in zip(("sample", "build", "forward", "backward", "sgd"), phase_us)},
        "algorithmic_bytes": {"forward": fwd_bytes, "backward": bwd_bytes, "sgd": sgd_bytes, "touched_rows": u_last},
        "loss_last_step": loss_last,
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        n = args.cpu_steps
        if n <= 0:
            v1, _, dt1 = cpu_baseline(wl, h, r, t, tabs, 1)
            n = max(2, min(60, int(15.0 / max(dt1, 1e-3))))
        v, done, cdt = cpu_baseline(wl, h, r, t, tabs, n)
        out["cpu_baseline"] = {"value": round(v, 1), "unit": "triplets/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {done} steps of the same workload (sampling, incidence build, "
                                         f"forward, backward, sgd), {cdt:.1f} s, single thread"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
