#!/usr/bin/env python3
"""Benchmark of the sparse-incidence KGE training step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic triplets that already sit in
HBM: negative sampling, incidence build (A and sorted A^T), forward (gather product + model projection
+ distance + margin-ranking loss), backward (transposed products) and the sparse SGD update.  Steps
walk the workload's batches in stored order, epoch after epoch (the last batch of an epoch is
partial).  Default workload: "mid" = TransE, d = 128, fp32, the configuration the headline metric is
quoted on.

Prints ONE JSON line; kernel_work() below holds the byte model behind "roofline".
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
MFMA_BF16_PEAK_TFLOPS = 2500.0
# kernels that run TransR products on the matrix cores, and how many products of 2*rows*d*k flops each runs
TRANSR_PRODUCTS = {"k_transr_fused": 2, "k_transr_project": 1, "k_transr_gx": 1, "k_transr_dm": 1}

# The kernel whose roofline is reported: the one with the largest share of GPU time in the
# rocprofv3 kernel trace of the same command (profiles/).
DOMINANT = {"mid": "k_seg_reduce", "tiny": "k_seg_reduce", "toruse": "k_seg_reduce", "transh": "k_seg_reduce",
            "transr": "k_transr_fused", "paper_transe": "k_seg_reduce", "paper_toruse": "k_seg_reduce",
            "paper_transr": "k_transr_fused"}
# ... without the look-ahead (--no-lookahead) the forward pass and the first scatter pass share the longest launch
DOMINANT_PLAIN = dict(DOMINANT, mid="k_fwd_scatter", tiny="k_fwd_scatter")
# ... and when the step is made of the separate calls (--api fused | separate)
DOMINANT_CALLS = {"mid": "k_seg_reduce", "tiny": "k_seg_reduce", "toruse": "k_seg_reduce", "transh": "k_forward_transh",
                  "transr": "k_transr_fused", "paper_transe": "k_seg_reduce", "paper_toruse": "k_seg_reduce",
                  "paper_transr": "k_transr_fused"}


# HBM bytes per launch of those kernels, measured: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (separate runs),
# each scaled by what the same counter reads for the library's plain copy kernel (FETCH_SIZE x2.0, WRITE_SIZE
# x1.0); the runs and their numbers are in profiles/<workload>_kernel_trace.txt and profiles/copy_calibration.txt.
# A different kernel (--kernel) or workload has no measured figure here and reports null.
# Keys: (workload, kernel, fused step or not).
TRAFFIC_BYTES = {("toruse", "k_seg_reduce", True): 1133.94e6 + 623.18e6,
                 ("toruse", "k_forward_stacked", True): 684.45e6 + 53.52e6,
                 ("toruse", "k_forward_stacked", False): 693.55e6 + 53.52e6,
                 ("toruse", "k_seg_reduce", False): 561.76e6 + 532.18e6,
                 ("toruse", "k_sgd_rows", False): 1056.94e6 + 526.37e6,
                 # mean of the two batches of an epoch (393,216 and 89,926 positives), like the timed mean
                 ("paper_transe", "k_seg_reduce", True): (9761.85e6 + 104.19e6 + 2281.04e6 + 99.90e6) / 2,
                 # with the look-ahead (the next batch's first build kernels ride in these launches)
                 ("mid", "k_seg_reduce", "rides"): 28.04e6 + 17.01e6,
                 ("mid", "k_fwd_scatter", "rides"): 27.44e6 + 9.25e6,
                 ("mid", "k_seg_fixup", "rides"): 3.67e6 + 0.42e6,
                 ("transh", "k_seg_reduce", "rides"): 142.54e6 + 14.81e6,
                 ("transh", "k_fwdh_scatter", "rides"): 34.67e6 + 105.22e6,
                 ("transh", "k_seg_fixup", "rides"): 4.06e6 + 0.48e6,
                 ("transr", "k_transr_fused", "rides"): 40.20e6 + 52.83e6,
                 ("transr", "k_seg_reduce", "rides"): 89.66e6 + 31.35e6,
                 ("transr", "k_seg_fixup", "rides"): 9.78e6 + 1.26e6,
                 # the other modes (profiles/semiring_complex_*_kernel_trace.txt, profiles/rank_mid_kernel_trace.txt)
                 ("semiring complex", "mid", "k_semiring_terms"): 66.64e6 + 100.66e6,
                 ("semiring complex", "toruse", "k_semiring_terms"): 1560.16e6 + 2013.27e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="mid", help="workload: tiny | mid | transh | transr | toruse | paper_transe | paper_toruse | paper_transr")
    ap.add_argument("--kernel", default=None, help="kernel to time for the roofline entry (default: the dominant one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--api", default="step", choices=["step", "fused", "separate"],
                    help="step: one stx_train_step call per step (default); fused: sample, build, forward, "
                         "stx_backward_sgd; separate: sample, build, forward, backward, sgd_step")
    ap.add_argument("--no-lookahead", action="store_true",
                    help="--api step: do not tell a step which batch follows (its first build kernel then runs on its own "
                         "instead of inside the previous step's transposed product)")
    ap.add_argument("--windows", type=int, default=5,
                    help="timed regions of --steps steps each; `value` is the median one, mean / median / min are printed")
    ap.add_argument("--no-hbm-leg", action="store_true",
                    help="default run (mid, --api step) only: leave out the short run of the HBM-resident configuration")
    ap.add_argument("--no-build-rates", action="store_true",
                    help="leave out the untimed pass that times negative sampling and the incidence build by themselves")
    ap.add_argument("--all-kernels", action="store_true",
                    help="extra untimed pass that brackets every kernel with events and adds 'kernels_us' to the output")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run the library's plain copy kernel 20 times on MIB MiB "
                         "(for scaling rocprofv3 byte counters) and exit")
    ap.add_argument("--cpu-steps", type=int, default=0, help="oracle steps to time (0 = pick for ~10-20 s)")
    ap.add_argument("--rank", action="store_true",
                    help="instead of the training step, time link prediction (stx_rank, tail and head side) of "
                         "--rank-queries test triplets against all entities of the workload's table")
    ap.add_argument("--rank-queries", type=int, default=0,
                    help="test triplets (default: 59,071, the size of FB15k's test split; 20,466, FB15k-237's, for TransR)")
    ap.add_argument("--semiring", default=None, choices=["distmult", "complex", "rotate"],
                    help="instead of the training step, time the semiring product of that model and its backward "
                         "(stx_spmm_semiring + stx_spmm_semiring_t) on the first batch of the workload's graph")
    return ap.parse_args()


def kernel_work(wl, kernel, rows, touched, fused=False, rides=False, segw=False):
    """Algorithmic work of ONE launch of `kernel` on a full batch: (amount, unit, bound, peak).
    row = 4*dim bytes.  rows = b*(1+k) matrix rows, nnz = 3*rows, touched = distinct columns.
    rides: the launch of the forward pass and the sort's last scatter pass (k_fwd_scatter, k_fwdh_scatter) also
    runs the next batch's k_emit (about 28 B per entry: indices in, CSR arrays, keys and negatives out), that of
    k_seg_reduce its first scatter pass (16 B per entry), that of k_seg_fixup the histogram pass of its second
    digit (4 B per entry).
    With TransR (both widths at most 128) the launch of k_seg_reduce also runs the dL/dM_r product and that of
    k_seg_fixup the sums of its partial matrices.
    segw: the launch of k_seg_reduce also runs the last kernel of this batch's build (sorted key and payload in,
    segment, row, packed entry and sign out: 21 B per entry)."""
    row = 4 * wl.dim
    nnz = 3 * rows
    if kernel == "k_seg_reduce" and (rides or segw):
        w, unit, bound, peak = kernel_work(wl, kernel, rows, touched, fused, False, False)
        if rides and wl.model == "transr" and wl.dim <= 128 and wl.rel_dim <= 128:
            w += kernel_work(wl, "k_transr_dm", rows, touched)[0]      # TransR's dL/dM_r product rides here too
        return w + nnz * ((16 if rides else 0) + (21 if segw else 0)), unit, bound, peak
    if kernel in ("k_fwd_scatter", "k_fwdh_scatter") and rides:
        w, unit, bound, peak = kernel_work(wl, kernel, rows, touched, fused, False, False)
        return w + nnz * 28, unit, bound, peak
    if kernel == "k_seg_fixup" and rides:
        return nnz * 4, "GB/s", "hbm", HBM_PEAK_GBS
    if kernel in ("k_fwd_hist", "k_fwdh_hist"):      # the forward pass and a histogram pass (4 B per key) in one launch
        w, unit, bound, peak = kernel_work(wl, "k_forward_stacked" if kernel == "k_fwd_hist" else "k_forward_transh", rows,
                                           touched, fused, False)
        return w + nnz * 4, unit, bound, peak
    if kernel == "k_scatter_finish":
        return nnz * 16, "GB/s", "hbm", HBM_PEAK_GBS
    packed = wl.model in ("transe", "toruse") and wl.dist in ("l1", "torus_l1")
    grow = (wl.dim // 4 + 4) if packed else row     # a stored dL/dx row: coefficient + sign bytes, or dense fp32
    if kernel == "k_forward_stacked" and wl.model in ("transe", "toruse"):
        # 3 gathered table rows + 12 B of column ids per row in; dL/dx row + score out
        return rows * (3 * row + 12 + grow + 4), "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_fwd_scatter":      # the same forward pass and one scatter pass of the sort in one launch
        return rows * (3 * row + 12 + grow + 4) + nnz * 16, "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_fwdh_scatter":     # TransH forward (below) and one scatter pass
        return rows * (2 * row + 2 * row / (1 + wl.n_neg) + 12 + 3 * row + 4) + nnz * 16, "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_forward_stacked":   # TransR: y row in, dL/dy row out, score out
        return rows * (2 * 4 * wl.rel_dim + 4), "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_forward_transh":
        # 2 entity rows per row, w_r and d_r once per positive, 12 B of ids in; gx, gy, gw rows + score out
        return rows * (2 * row + 2 * row / (1 + wl.n_neg) + 12 + 3 * row + 4), "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_seg_reduce":
        # one source row + 4 B packed entry per sorted entry in, one row per column out, over all 3*rows entries
        if wl.model == "transh":   # both products (all entries -> dE, d(d_r); relation entries -> dw_r) in one launch
            out_rows = (touched + min(wl.n_rel, rows)) * row * (2 if fused else 1)   # fused: table row in, table row out
            return nnz * (row + 4) + rows * (row + 4) + out_rows, "GB/s", "hbm", HBM_PEAK_GBS
        if wl.model == "transr":   # one launch when dim == rel_dim
            return nnz * (row + 4) + touched * row * (2 if fused else 1), "GB/s", "hbm", HBM_PEAK_GBS
        if fused and wl.model in ("transe", "toruse"):
            # fused update: the table row is read and written where the gradient row would have been written
            return nnz * (grow + 4) + touched * 2 * row, "GB/s", "hbm", HBM_PEAK_GBS
        return nnz * (grow + 4) + touched * row, "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_sgd_rows":
        return touched * 3 * row, "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_semiring":          # three gathered rows + ids in, the product row out
        return rows * (3 * row + 12 + row), "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_semiring_terms":    # three gathered rows, the dL/dZ row and ids in, three term rows out
        return rows * (4 * row + 12 + 3 * row), "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_seg_reduce_terms":  # the transposed product over the term rows: one row per entry in, one per column out
        return nnz * (row + 4) + touched * row, "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_scatter":
        return nnz * 16, "GB/s", "hbm", HBM_PEAK_GBS      # key + payload in, key + payload out
    # TransR's three products: 2*d*k flop per row against ~2 KB of row traffic is ~20 flop per byte, far left of
    # the ridge (2.5 PFLOP/s / 8 TB/s = 312 flop per byte): their roofline is the memory one.  Bytes: the gathered
    # fp32 rows, the fp32 rows written, the bf16 transposed tiles, and the bf16 copy of M_r once per relation.
    nrel = min(wl.n_rel, rows)
    if kernel == "k_transr_fused":     # forward product, distances, hinge and GX product on one staged tile:
        # h and t rows and 12 B of ids in; dL/dy row, dL/dx row, both bf16 tiles and the score out; both copies of M_r
        return (rows * (2 * row + 12 + 4 * wl.rel_dim + row + 2 * wl.dim + 2 * wl.rel_dim + 4)
                + nrel * 4 * wl.dim * wl.rel_dim), "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_transr_project":   # h and t rows, 12 B of ids, y row out, x tile out
        return rows * (2 * row + 12 + 4 * wl.rel_dim + 2 * wl.dim) + nrel * 2 * wl.dim * wl.rel_dim, "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_transr_gx":        # dL/dy row in, dL/dx row out, dL/dy tile out
        return rows * (4 + 4 * wl.rel_dim + row + 2 * wl.rel_dim) + nrel * 2 * wl.dim * wl.rel_dim, "GB/s", "hbm", HBM_PEAK_GBS
    if kernel == "k_transr_dm":        # both tiles in, dL/dM_r out
        return rows * (2 * wl.rel_dim + 2 * wl.dim) + nrel * 4 * wl.dim * wl.rel_dim, "GB/s", "hbm", HBM_PEAK_GBS
    raise ValueError(kernel)


def kernel_min_bytes(wl, kernel, rows, touched, fused=False):
    """Lower bound on the bytes one launch must move: every distinct table row once instead of once per entry
    that names it, every stored dL/dx row once.  None for kernels without such a bound here."""
    row = 4 * wl.dim
    nnz = 3 * rows
    packed = wl.model in ("transe", "toruse") and wl.dist in ("l1", "torus_l1")
    grow = (wl.dim // 4 + 4) if packed else row
    stacked = wl.model in ("transe", "toruse")
    if kernel in ("k_forward_stacked", "k_fwd_scatter") and stacked:
        return touched * row + rows * (12 + grow + 4) + (nnz * 16 if kernel == "k_fwd_scatter" else 0)
    if kernel == "k_seg_reduce" and stacked:
        return rows * grow + nnz * 4 + touched * row * (2 if fused else 1)
    return None


def cpu_baseline(wl, h, r, t, tabs, n_steps):
    """The CPU oracle as it stands, single thread, on the first batches of the same workload."""
    from oracle import stxo
    from tests.util import oracle_batch, oracle_config, oracle_tables
    cfg = oracle_config(wl)
    tb = oracle_tables(tabs)
    slices = [(s, min(s + wl.batch, wl.n_triplets)) for s in range(0, wl.n_triplets, wl.batch)]
    rows = done = 0
    t0 = time.perf_counter()
    for i in range(n_steps):
        lo, hi = slices[i % len(slices)]
        bt = oracle_batch(wl, h, r, t, lo, hi)
        stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
        stxo.train_step(cfg, tb, bt, wl.lr)
        rows += bt.rows
        done += 1
    dt = time.perf_counter() - t0
    return rows / dt, done, dt


# Vector-ALU peak in operations: 256 compute units x 128 fp32 lanes x 2.4 GHz = 78.6 T operations per second; the
# published 157.3 TFLOP/s counts every one of them as a fused multiply-add, i.e. two flops.  A sum of absolute
# differences has no product to fuse, so its flop peak is the operation peak.
VALU_OPS_PEAK_T = 256 * 128 * 2.4e9 / 1e12
# vector operations per (query, candidate, row element) in k_rank, and flops they stand for
RANK_OPS = {"l1": (2, 2), "l2": (2, 3), "l2_sq": (2, 3), "torus_l1": (5, 5), "torus_l2": (5, 6)}
# TransH (k_rank_h): a fused multiply-add for w.e in the first pass over the row, then a difference, a fused
# multiply-add for the projection and the distance step
RANK_OPS_H = {"l1": (4, 6), "l2": (4, 7), "l2_sq": (4, 7), "torus_l1": (7, 9), "torus_l2": (7, 10)}


def bench_rank(args, wl, dev):
    """One evaluation pass: tail and head ranking of every test triplet against all entities."""
    import numpy as np
    import torch

    from paper_2502_16949_amd import binding as B
    from paper_2502_16949_amd import workloads as W
    nq = args.rank_queries or (20_466 if wl.model == "transr" else W.N_TEST_FB15K)
    h, r, t = W.make_test_triplets(wl, nq)
    tabs = W.make_tables(wl)
    transh, transr = wl.model == "transh", wl.model == "transr"
    cfg = B.make_config(wl.model, wl.dist, wl.n_ent, wl.n_rel, wl.dim, 8, 1, rel_dim=wl.rel_dim, margin=wl.margin,
                        flags=B.STX_FLAG_BF16_PROJ if transr else 0)
    ctx = B.Context(cfg, dev)
    params = B.Params(*(None if tabs.get(k) is None else torch.from_numpy(tabs[k]).to(dev) for k in ("ent", "rel", "w", "proj")))
    need = B.stx_rank_work_bytes(ctx, nq)
    work = torch.empty(need + 256, dtype=torch.uint8, device=dev) if need else None
    rank_kernel = "k_rank_h" if transh else "k_rank"
    hd, rd, td = (torch.from_numpy(a).to(dev) for a in (h, r, t))
    ts = torch.empty(2, nq, dtype=torch.float32, device=dev)
    less = torch.empty(2, nq, dtype=torch.int32, device=dev)
    equal = torch.empty(2, nq, dtype=torch.int32, device=dev)

    def step():
        B.stx_rank(ctx, params, hd, rd, td, B.STX_TAIL, ts[0], less[0], equal[0], work)
        B.stx_rank(ctx, params, hd, rd, td, B.STX_HEAD, ts[1], less[1], equal[1], work)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.stx_profile_kernel(ctx, rank_kernel, 2 * args.steps * (wl.n_rel if transr else 1))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_us, kernel_n = B.stx_profile_read(ctx)
    ops, flops = (RANK_OPS_H if transh else RANK_OPS)[wl.dist]
    # per side; TransR sweeps rows of rel_dim projected values in one launch per relation: the launches of a
    # side are priced together (mean launch time x launches per side)
    elems = float(nq) * wl.n_ent * (wl.rel_dim if transr else wl.dim)
    side_us = kernel_us * kernel_n / (2 * args.steps) if args.steps else 0.0
    achieved = elems * flops / (side_us * 1e-6) / 1e12 if side_us > 0 else 0.0
    peak = VALU_OPS_PEAK_T * flops / ops
    best = 1 + less.cpu().numpy().astype(np.int64)
    out = {"metric": f"link prediction, test triplets ranked/sec (tail and head, all {wl.n_ent} entities) {wl.model} "
                     f"{wl.dist} d={wl.dim} fp32",
           "value": round(nq * args.steps / dt, 1), "unit": "triplets/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{wl.name} tables ({wl.n_ent} entities, {wl.n_rel} relations, dim {wl.dim}, {wl.dist}), "
                                  f"{nq} test triplets (the size of the test split of FB15k{'-237' if transr else ''}) from the "
                                  "graph's degree laws",
                      "step": "stx_rank tail side + stx_rank head side over all test triplets"},
           "hits_at_10_raw": round(float((best <= 10).mean()), 4),
           "roofline": {"bound": "alu", "kernel": rank_kernel, "achieved": round(achieved, 2), "peak": round(peak, 1),
                        "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": None,
                        "work_per_launch": int(elems * flops), "avg_launch_us": round(kernel_us, 2),
                        "launches_per_step": round(kernel_n / args.steps, 2),
                        "note": f"{ops} vector operations ({flops} flops) per query x candidate x element; peak = 256 CUs x "
                                "128 lanes x 2.4 GHz operations per second"}}
    if not args.no_cpu_baseline:
        from oracle import stxo
        from tests.util import oracle_config
        ocfg = oracle_config(wl)
        otab = stxo.Tables(tabs["ent"], tabs.get("rel"), tabs.get("w"), tabs.get("proj"))
        if transr:
            ocfg = oracle_config(wl, bf16=False)
        n = 2 if transr else 8
        while True:
            t0 = time.perf_counter()
            stxo.rank(ocfg, otab, h[:n], r[:n], t[:n], stxo.TAIL)
            stxo.rank(ocfg, otab, h[:n], r[:n], t[:n], stxo.HEAD)
            cdt = time.perf_counter() - t0
            if cdt >= 8.0 or n >= nq:
                break
            n = min(nq, max(n * 2, int(n * 12.0 / max(cdt, 1e-3))))
        out["cpu_baseline"] = {"value": round(n / cdt, 2), "unit": "triplets/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {n} test triplets, both sides, {cdt:.1f} s, single thread"}
    print(json.dumps(out))


def bench_semiring(args, wl, dev):
    """Forward and backward of one semiring product (Appendix D) over the rows of one batch."""
    import numpy as np
    import torch

    from paper_2502_16949_amd import binding as B
    from paper_2502_16949_amd import workloads as W
    kind = {"distmult": B.STX_DISTMULT, "complex": B.STX_COMPLEX, "rotate": B.STX_ROTATE}[args.semiring]
    h, r, t = W.make_graph(wl)
    tabs = W.make_tables(wl)
    b = min(wl.batch, wl.n_triplets)
    hd, rd, td = (torch.from_numpy(a[:b].copy()).to(dev) for a in (h, r, t))
    cfg = B.make_config("transe", "l2", wl.n_ent, wl.n_rel, wl.dim, b, wl.n_neg, margin=wl.margin)
    ctx = B.Context(cfg, dev)
    ent = tabs["ent"] if tabs["ent"].shape[0] == wl.n_ent + wl.n_rel else np.concatenate([tabs["ent"], tabs["rel"]])
    params = B.Params(torch.from_numpy(np.ascontiguousarray(ent[:, :wl.dim])).to(dev))
    inc, grads = B.Incidence(ctx), B.Grads(ctx)
    nh = torch.empty(b * wl.n_neg, dtype=torch.int32, device=dev)
    nt = torch.empty_like(nh)
    B.stx_sample_negatives(ctx, hd, rd, td, wl.n_neg, W.negative_seed(wl), 0, wl.n_triplets, 0, nh, nt)
    B.stx_build_incidence(ctx, hd, rd, td, nh, nt, wl.n_neg, inc)
    rows = inc.n_rows
    z = torch.empty(rows, wl.dim, dtype=torch.float32, device=dev)
    gz = torch.rand(rows, wl.dim, dtype=torch.float32, device=dev) - 0.5
    work = torch.empty(3 * rows * wl.dim, dtype=torch.float32, device=dev)
    kernel = args.kernel or "k_semiring_terms"
    for _ in range(args.warmup):
        B.stx_spmm_semiring(ctx, inc, params, kind, z)
        B.stx_spmm_semiring_t(ctx, inc, params, kind, gz, work, grads)
    torch.cuda.synchronize()
    B.stx_profile_kernel(ctx, kernel, 4 * args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        B.stx_spmm_semiring(ctx, inc, params, kind, z)
        B.stx_spmm_semiring_t(ctx, inc, params, kind, gz, work, grads)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_us, kernel_n = B.stx_profile_read(ctx)
    u = int(inc.n_touched.item())
    work_b, unit, bound, peak = kernel_work(wl, "k_seg_reduce_terms" if kernel == "k_seg_reduce" else kernel, rows, u)
    achieved = work_b / (kernel_us * 1e-6) / 1e9 if kernel_us > 0 else 0.0
    n_ph = min(args.steps, 40)
    B.stx_profile_kernel(ctx, "*", 8 * n_ph)
    for _ in range(n_ph):
        B.stx_spmm_semiring(ctx, inc, params, kind, z)
        B.stx_spmm_semiring_t(ctx, inc, params, kind, gz, work, grads)
    kernels_us = {k: [round(v[0], 2), round(v[1] / n_ph, 2)] for k, v in B.stx_profile_dump(ctx).items()}
    out = {"metric": f"semiring product rows/sec ({args.semiring}: forward + backward) d={wl.dim} fp32",
           "value": round(rows * args.steps / dt, 1), "unit": "rows/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{wl.name} graph, first batch: {rows} rows, {u} touched columns, dim {wl.dim}",
                      "step": "stx_spmm_semiring + stx_spmm_semiring_t"},
           "roofline": {"bound": bound, "kernel": kernel, "achieved": round(achieved, 1), "peak": peak, "unit": unit,
                        "frac": round(achieved / peak, 4),
                        "traffic": TRAFFIC_BYTES.get((f"semiring {args.semiring}", wl.name, kernel)),
                        "work_per_launch": int(work_b),
                        "avg_launch_us": round(kernel_us, 2), "launches_per_step": round(kernel_n / args.steps, 2)},
           "kernels_us": kernels_us}
    if not args.no_cpu_baseline:
        from oracle import stxo
        from tests.util import oracle_batch
        bt = oracle_batch(wl, h, r, t, 0, b)
        oinc = stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
        okind = {"distmult": stxo.DISTMULT, "complex": stxo.COMPLEX, "rotate": stxo.ROTATE}[args.semiring]
        gzn = gz.cpu().numpy()
        n, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < 10.0:
            stxo.spmm_semiring(oinc.colidx, ent, okind)
            stxo.spmm_semiring_t(oinc.colidx, ent, okind, gzn)
            n += 1
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(rows * n / cdt, 1), "unit": "rows/s", "cores": 1, "kind": "oracle",
                               "sample": f"{n} forward + backward passes over the same batch, {cdt:.1f} s, single thread"}
    print(json.dumps(out))


# Last-level cache of the part (the memory-side Infinity Cache): a working set below it is served from cache after
# the first touch, and a "fraction of the HBM peak" is then a nominal figure.
LLC_BYTES = 256 << 20


def host_info():
    model = "unknown"
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                model = ln.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {"nproc": os.cpu_count() or 1, "usable_cores": usable, "cpu_model": model}


def roof_of(wl, kernel, us):
    """Which roof a kernel's byte figure can meaningfully be held against."""
    table = (wl.n_ent + wl.n_rel) * wl.dim * 4
    packed = wl.model in ("transe", "toruse") and wl.dist in ("l1", "torus_l1")
    g = wl.rows_per_batch * ((wl.dim // 4 + 4) if packed else 4 * wl.dim * (3 if wl.model in ("transh", "transr") else 1))
    if table + g > LLC_BYTES:
        return "hbm: the working set (%.0f MB of tables and per-row buffers) exceeds the %d MB last-level cache" % (
            (table + g) / 1e6, LLC_BYTES >> 20)
    if us < 12.0 and kernel in ("k_seg_fixup", "k_scatter", "k_scatter_finish", "k_hist_finish", "k_emit", "k_finish_loss"):
        return "latency: a few dependent memory round trips on little data; bytes per second say nothing here"
    return ("cache: tables and per-row buffers (%.0f MB) stay in the %d MB last-level cache, so the algorithmic bytes are "
            "mostly not HBM traffic and the fraction of the HBM peak is nominal" % ((table + g) / 1e6, LLC_BYTES >> 20))


class Job:
    """One workload set up on the GPU: context, tables, marshalled argument lists of every batch."""

    def __init__(self, wl, dev, api, lookahead):
        import ctypes as C

        import torch

        from paper_2502_16949_amd import binding as B
        from paper_2502_16949_amd import workloads as W
        self.wl, self.api, self.B, self.torch = wl, api, B, torch
        self.fused = api != "separate"
        self.one_call = api == "step"
        # batches whose first build kernels can run inside the previous step's launches (see stx_batch.next)
        self.rides = (self.one_call and lookahead and (wl.model != "transr" or wl.n_rel <= 4096)
                      and wl.n_ent + wl.n_rel <= 65536 and 3 * wl.rows_per_batch <= (1 << 19) and wl.dim <= 256)
        # the one-call step leaves the last kernel of the build to the launch of the transposed product (rows of
        # one float4 per lane; TransR when its work items come from the rows-per-relation counts)
        self.segw = self.one_call and (wl.model != "transr" or wl.n_rel <= 4096) and wl.dim <= 256
        self.h, self.r, self.t = W.make_graph(wl)
        self.tabs = W.make_tables(wl)
        hd, rd, td = (torch.from_numpy(a).to(dev) for a in (self.h, self.r, self.t))
        flags = {"transh": B.STX_FLAG_RENORM_W, "transr": B.STX_FLAG_BF16_PROJ}.get(wl.model, 0)
        cfg = B.make_config(wl.model, wl.dist, wl.n_ent, wl.n_rel, wl.dim, wl.batch, wl.n_neg, rel_dim=wl.rel_dim,
                            margin=wl.margin, flags=flags)
        self.ctx = ctx = B.Context(cfg, dev)
        self.params = params = B.Params(*(None if self.tabs.get(k) is None else torch.from_numpy(self.tabs[k]).to(dev)
                                          for k in ("ent", "rel", "w", "proj")))
        self.inc = inc = B.Incidence(ctx)
        self.grads = grads = B.Grads(ctx)
        self.scores = scores = torch.empty(ctx.rows_max, dtype=torch.float32, device=dev)
        self.loss = loss = torch.zeros(1, dtype=torch.float32, device=dev)
        nh = torch.empty(wl.batch * wl.n_neg, dtype=torch.int32, device=dev)
        nt = torch.empty(wl.batch * wl.n_neg, dtype=torch.int32, device=dev)
        self.keep = (hd, rd, td, nh, nt)
        self.slices = W.batch_slices(wl)
        seed = W.negative_seed(wl)
        byref = C.byref
        self.L = B.lib()

        # Argument lists are marshalled once per batch; the timed loop makes only the C calls.
        def marshal(lo, hi):
            hb, rb, tb = (a.data_ptr() + 4 * lo for a in (hd, rd, td))
            b = hi - lo
            return ((ctx.handle, hb, rb, tb, b, wl.n_neg, seed, 0, wl.n_triplets, lo, nh.data_ptr(), nt.data_ptr()),
                    (ctx.handle, hb, rb, tb, nh.data_ptr(), nt.data_ptr(), b, wl.n_neg, byref(inc.c)),
                    (ctx.handle, byref(inc.c), byref(params.c), scores.data_ptr(), loss.data_ptr()),
                    (ctx.handle, byref(inc.c), byref(params.c), byref(grads.c)),
                    (ctx.handle, byref(params.c), byref(inc.c), byref(grads.c), wl.lr),
                    (ctx.handle, byref(inc.c), byref(params.c), byref(grads.c), wl.lr),
                    (ctx.handle, byref(B.make_batch(hd[lo:hi], rd[lo:hi], td[lo:hi], wl.n_neg, seed, 0, wl.n_triplets, lo,
                                                    nh, nt)),
                     byref(inc.c), byref(params.c), byref(grads.c), wl.lr, scores.data_ptr(), loss.data_ptr()),
                    b * (1 + wl.n_neg))
        self.calls = [marshal(lo, hi) for lo, hi in self.slices]
        if self.one_call and lookahead:
            # every step names the batch of the step after it (steps walk the batches cyclically)
            B.link_batches([c[6][1]._obj for c in self.calls], cyclic=True)
        self.next_step = 0

    def step(self, ev=None):
        """The next step of the walk over the batches; returns its number of matrix rows."""
        i = self.next_step
        self.next_step += 1
        L = self.L
        a_s, a_b, a_f, a_g, a_u, a_bu, a_step, rows = self.calls[i % len(self.calls)]
        if self.one_call:
            if L.stx_train_step(*a_step):
                raise RuntimeError(f"stx_train_step failed in step {i}")
            return rows
        if ev: ev[0].record()
        st = L.stx_sample_negatives(*a_s)
        if ev: ev[1].record()
        st |= L.stx_build_incidence(*a_b)
        if ev: ev[2].record()
        st |= L.stx_forward(*a_f)
        if ev: ev[3].record()
        if self.fused:
            st |= L.stx_backward_sgd(*a_bu)
            if ev: ev[4].record()
        else:
            st |= L.stx_backward(*a_g)
            if ev: ev[4].record()
            st |= L.stx_sgd_step(*a_u)
        if ev: ev[5].record()
        if st:
            raise RuntimeError(f"a library call failed in step {i} (or-ed status {st})")
        return rows

    def run(self, n):
        rows = 0
        for _ in range(n):
            rows += self.step()
        return rows

    def timed_windows(self, steps, windows):
        """`windows` regions of exactly `steps` steps, each between two device synchronisations, with nothing
        else on the stream (no event brackets).  Returns [(seconds, rows, host seconds to enqueue)]."""
        out = []
        for _ in range(windows):
            self.torch.cuda.synchronize()
            t0 = time.perf_counter()
            rows = self.run(steps)
            t_enq = time.perf_counter() - t0
            self.torch.cuda.synchronize()
            out.append((time.perf_counter() - t0, rows, t_enq))
        return out

    def bracketed(self, name, steps, cap_per_step=40):
        """Untimed pass: `steps` more steps with the launches of kernel `name` ("*": every kernel) bracketed by HIP
        events on the library's stream.  Returns ({kernel: (mean us, launches per step)}, mean rows per step)."""
        B = self.B
        B.stx_profile_kernel(self.ctx, name, cap_per_step * steps)
        rows = self.run(steps)
        if name == "*":
            got = {k: (v[0], v[1] / steps) for k, v in B.stx_profile_dump(self.ctx).items()}
        else:
            us, n = B.stx_profile_read(self.ctx)
            got = {name: (us, n / steps)}
        B.stx_profile_kernel(self.ctx, None, 0)
        return got, rows / steps

    def phases(self, steps):
        """Separate calls only: mean microseconds of each call of a step (events on the current stream)."""
        torch = self.torch
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(steps)]
        rows = 0
        for ev in events:
            rows += self.step(ev)
        torch.cuda.synchronize()
        tot = [0.0] * 5
        for ev in events:
            for p in range(5):
                tot[p] += ev[p].elapsed_time(ev[p + 1])
        names = ("sample", "build", "forward", "backward_sgd" if self.fused else "backward", "sgd")
        return {k: v / steps * 1e3 for k, v in zip(names, tot)}, rows / steps

    def kernel_entry(self, kname, us, mean_rows, touched):
        """Roofline entry of one kernel from its mean launch time: algorithmic bytes, the fewest bytes the launch
        could move, the measured traffic where a profile has it, and the roof the figures are held against."""
        wl = self.wl
        u = touched * mean_rows / wl.rows_per_batch
        w, unit, bound, peak = kernel_work(wl, kname, mean_rows, u, self.fused, self.rides, self.segw)
        ach = w / (us * 1e-6) / (1e9 if unit == "GB/s" else 1e12) if us > 0 else 0.0
        e = {"bound": bound, "kernel": kname, "achieved": round(ach, 1), "peak": peak, "unit": unit,
             "frac": round(ach / peak, 4),
             "traffic": TRAFFIC_BYTES.get((wl.name, kname, "rides" if self.rides else self.fused)),
             "work_per_launch": int(w), "avg_launch_us": round(us, 2), "roof": roof_of(wl, kname, us)}
        bmin = kernel_min_bytes(wl, kname, mean_rows, u, self.fused)
        if bmin is not None and us > 0:
            e["min_bytes_per_launch"] = int(bmin)
            e["achieved_min_bytes"] = round(bmin / (us * 1e-6) / 1e9, 1)
        if e["traffic"] and us > 0:
            e["achieved_traffic"] = round(e["traffic"] / (us * 1e-6) / 1e9, 1)
        if ach > peak and kname in ("k_forward_stacked", "k_fwd_scatter"):
            # the algorithmic figure counts three gathered table rows per matrix row; the kernel requests a positive's
            # rows once for all of its negatives and repeated rows come from the caches
            e["note"] = ("above the peak because the algorithmic bytes (three table rows per matrix row) are more than "
                         "this kernel moves: it fetches a positive's rows once for its negatives and hot rows hit in "
                         "cache; hold it against achieved_traffic and achieved_min_bytes instead")
        return e


def summarize(windows, steps):
    ms = sorted(w[0] / steps * 1e3 for w in windows)
    n = len(ms)
    med = ms[n // 2] if n % 2 else 0.5 * (ms[n // 2 - 1] + ms[n // 2])
    return {"windows": n, "steps_per_window": steps, "ms_per_step_mean": round(sum(ms) / n, 5),
            "ms_per_step_median": round(med, 5), "ms_per_step_min": round(ms[0], 5), "ms_per_step_max": round(ms[-1], 5)}


def median_window(windows):
    order = sorted(windows, key=lambda w: w[0] / max(w[1], 1))
    return order[(len(order) - 1) // 2]


def hbm_resident_leg(args, dev):
    """The HBM-resident configuration ("toruse": 2 GB table, 1.3 M rows per batch) on the same line as the headline:
    a short run of linked stx_train_step calls, then untimed bracketed passes for the kernels the 60 % target is
    about: the fused transposed product, the forward gather, and the stand-alone update (separate calls)."""
    import torch

    from paper_2502_16949_amd import workloads as W
    wl = W.WORKLOADS["toruse"]
    steps, warm = max(20, min(args.steps, 40)), 5
    job = Job(wl, dev, "step", True)
    job.run(warm)
    wins = job.timed_windows(steps, 3)
    dt, rows, _ = median_window(wins)
    u = int(job.inc.n_touched.item())
    got, mean_rows = job.bracketed("*", 20)
    kernels = {}
    for kname in ("k_seg_reduce", "k_forward_stacked"):
        if kname in got:
            kernels[kname + (" (fused update)" if kname == "k_seg_reduce" else "")] = job.kernel_entry(kname, got[kname][0], mean_rows, u)
    leg = {"workload": f"toruse: toruse torus_l1, {wl.n_ent} entities, {wl.n_rel} relations, dim {wl.dim}, batch {wl.batch}, "
                       f"{wl.n_neg} negatives per positive ({wl.rows_per_batch} rows per step, {u} touched rows)",
           "value": round(rows / dt, 1), "unit": "triplets/s", "ms_per_step": round(dt / steps * 1e3, 4),
           "timing": summarize(wins, steps), "kernels_us": {k: [round(v[0], 2), round(v[1], 2)] for k, v in got.items()}}
    # the stand-alone update and the unfused product: the same batches through the separate calls
    del job
    torch.cuda.empty_cache()
    sep = Job(wl, dev, "separate", False)
    sep.run(3)
    got2, mean_rows2 = sep.bracketed("*", 10)
    u2 = int(sep.inc.n_touched.item())
    for kname in ("k_sgd_rows", "k_seg_reduce"):
        if kname in got2:
            kernels[kname + (" (gradient rows stored)" if kname == "k_seg_reduce" else "")] = sep.kernel_entry(kname, got2[kname][0], mean_rows2, u2)
    ph, _ = sep.phases(6)
    leg["separate_calls_us"] = {k: round(v, 1) for k, v in ph.items()}
    leg["kernels"] = kernels
    return leg


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
    if args.copy_calibration:
        copy_calibration(args, dev)
        return
    wl = W.WORKLOADS[args.config]
    if args.semiring:
        bench_semiring(args, wl, dev)
        return
    if args.rank:
        bench_rank(args, wl, dev)
        return
    kernel = args.kernel or ((DOMINANT_PLAIN if args.no_lookahead else DOMINANT) if args.api == "step"
                             else DOMINANT_CALLS)[wl.name]
    job = Job(wl, dev, args.api, not args.no_lookahead)
    job.run(args.warmup)

    # ---- timed region: windows of exactly --steps steps, each between two device synchronisations; nothing but
    # the steps is on the stream (no event brackets).  `value` is the median window. ---------------------------
    wins = job.timed_windows(args.steps, max(1, args.windows))
    dt, rows_done, t_enq = median_window(wins)
    loss_last = float(job.loss.item())
    u_last = int(job.inc.n_touched.item())

    # ---- untimed passes: the dominant kernel's launches bracketed by HIP events on the library's stream (its
    # roofline entry), then every kernel (where the time goes), then, for separate calls, the calls themselves ----
    n_ph = max(min(args.steps, 60), min(len(job.calls), 30))
    got, mean_rows = job.bracketed(kernel, n_ph)
    kernel_us, per_launch = got[kernel]
    roofline = job.kernel_entry(kernel, kernel_us, mean_rows, u_last)
    roofline["launches_per_step"] = round(per_launch, 2)
    if kernel == "k_seg_reduce" and (job.rides or job.segw):
        roofline["note"] = ("this launch also runs " +
                            " and ".join((["the last kernel of this batch's build (21 B per entry)"] if job.segw else []) +
                                         (["the first scatter pass of the next batch's sort (16 B per entry)"] if job.rides else [])) +
                            ", counted")
    if kernel in TRANSR_PRODUCTS and kernel_us > 0:
        # the same launch priced as a contraction, against the dense bf16 matrix-core peak
        tf = TRANSR_PRODUCTS[kernel] * 2.0 * mean_rows * wl.dim * wl.rel_dim / (kernel_us * 1e-6) / 1e12
        roofline["mfma"] = {"achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                            "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                            "counters": "profiles/transr_kernel_trace.txt (matrix-core busy cycles and operations from rocprofv3 --pmc)"}

    out = {
        "metric": "training triplets/sec (pos+neg) TransE d=128 fp32" if wl.name == "mid"
                  else f"training triplets/sec (pos+neg) {wl.model} d={wl.dim} fp32",
        "value": round(rows_done / dt, 1), "unit": "triplets/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if wl.model != "transr" else "f32 (bf16 MFMA operands)",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.model} {wl.dist}, {wl.n_ent} entities, {wl.n_rel} relations, "
                               f"{wl.n_triplets} triplets (Zipf {wl.zipf_ent}/{wl.zipf_rel}), dim {wl.dim}, "
                               f"batch {wl.batch}, {wl.n_neg} negative(s) per positive, margin {wl.margin}, "
                               f"SGD lr {wl.lr}",
                   "rows_per_full_batch": wl.rows_per_batch, "batches_per_epoch": len(job.slices),
                   "step": ("stx_train_step: sample negatives + build incidence + forward + backward with fused sgd, one call"
                            + ("" if args.no_lookahead else "; each call names the next batch") if job.one_call else "sample negatives + build incidence + forward + " +
                            ("backward with fused sgd (stx_backward_sgd)" if job.fused else "backward + sgd")),
                   "api": args.api},
        "timing": dict(summarize(wins, args.steps), value_is="the median window; no event brackets inside any window"),
        "host_enqueue_us_per_step": round(t_enq / args.steps * 1e6, 2),
        "touched_rows_last_step": u_last,
        "loss_last_step": loss_last,
        "roofline": roofline,
    }

    if not job.one_call:
        ph, ph_rows = job.phases(min(args.steps, 60))
        out["phase_us"] = {k: round(v, 2) for k, v in ph.items()}
    if args.all_kernels or job.one_call:
        # every kernel bracketed: [mean microseconds, launches per step] (a bracket adds 2-4 us to a kernel)
        allk, rows_k = job.bracketed("*", n_ph)
        out["kernels_us"] = {k: [round(v[0], 2), round(v[1], 2)] for k, v in allk.items()}
        others = {}
        for kname, (us, _) in allk.items():
            if kname == kernel or us <= 0:
                continue
            try:
                others[kname] = job.kernel_entry(kname, us, rows_k, u_last)
            except ValueError:
                continue
        out["roofline_other_kernels"] = others

    # ---- sampling and build throughput by themselves (untimed for the headline): the same batches through the
    # separate calls, each call between events -------------------------------------------------------------
    if not args.no_build_rates:
        if job.one_call:
            peak_bytes = torch.cuda.max_memory_allocated()
            aux = Job(wl, dev, "separate", False)
            aux.run(3)
        else:
            aux = job
        ph, ph_rows = aux.phases(min(max(args.steps, 10), 30))
        nneg = ph_rows * wl.n_neg / (1 + wl.n_neg)
        out["build_keys_per_s"] = round(3 * ph_rows / (ph["build"] * 1e-6), 1) if ph["build"] > 0 else None
        out["sample_negs_per_s"] = round(nneg / (ph["sample"] * 1e-6), 1) if ph["sample"] > 0 and nneg else None
        out["build_us"], out["sample_us"] = round(ph["build"], 2), round(ph["sample"], 2)
        if aux is not job:
            del aux
    out["peak_device_bytes"] = int(torch.cuda.max_memory_allocated())

    if not args.no_cpu_baseline:
        n = args.cpu_steps
        if n <= 0:
            _, _, dt1 = cpu_baseline(wl, job.h, job.r, job.t, job.tabs, 1)
            n = max(2, min(400, int(15.0 / max(dt1, 1e-3))))
        v, done, cdt = cpu_baseline(wl, job.h, job.r, job.t, job.tabs, n)
        out["cpu_baseline"] = dict({"value": round(v, 1), "unit": "triplets/s", "cores": 1, "kind": "oracle",
                                    "sample": f"first {done} steps of the same workload (sampling, incidence build, "
                                              f"forward, backward, sgd), {cdt:.1f} s, single thread"}, **host_info())

    # ---- the HBM-resident configuration beside the cache-resident headline ---------------------------------
    if wl.name == "mid" and args.api == "step" and not args.no_hbm_leg:
        del job
        torch.cuda.empty_cache()
        out["hbm_resident"] = hbm_resident_leg(args, dev)
    print(json.dumps(out))


def copy_calibration(args, dev):
    import torch

    from paper_2502_16949_amd import binding as B
    n = args.copy_calibration * (1 << 20) // 4
    cctx = B.Context(B.make_config("transe", "l1", 16, 1, 4, 1, 0), dev)
    src = torch.ones(n, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    for _ in range(20):
        B.stx_copy_f32(cctx, dst, src)
    # the second pattern: one 32-byte read per lane, slots 512 bytes apart, every slot once per launch
    n_slots = 4 * n // 512
    sink = torch.zeros(16384, dtype=torch.float32, device=dev)
    for _ in range(20):
        B.stx_read_sectors(cctx, src, n_slots, 512, n_slots, sink)
    torch.cuda.synchronize()
    print(json.dumps({"k_copy_f32": {"bytes_read": 4 * n, "bytes_written": 4 * n, "launches": 20},
                      "k_read_sectors": {"bytes_read": 32 * n_slots, "reads": n_slots, "slot_bytes": 512,
                                         "bytes_written": 0, "launches": 20}}))


if __name__ == "__main__":
    main()
