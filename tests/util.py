"""Shared helpers of the test-suite: workload -> oracle objects, small random problems."""
from __future__ import annotations

import numpy as np

from oracle import stxo
from paper_2502_16949_amd import workloads as W

MODEL = {"transe": stxo.TRANSE, "transh": stxo.TRANSH, "transr": stxo.TRANSR, "toruse": stxo.TORUSE}
DIST = {"l1": stxo.L1, "l2": stxo.L2, "torus_l1": stxo.TORUS_L1, "torus_l2": stxo.TORUS_L2, "l2_sq": stxo.L2_SQ}


def oracle_config(wl: W.Workload, reduce=stxo.SUM, bf16=None) -> stxo.Config:
    return stxo.Config(MODEL[wl.model], DIST[wl.dist], wl.n_ent, wl.n_rel, wl.dim, wl.rel_dim, wl.margin,
                       reduce, wl.bf16_proj if bf16 is None else bf16)


def oracle_tables(tabs: dict) -> stxo.Tables:
    return stxo.Tables(tabs["ent"].copy(), *(None if tabs.get(k) is None else tabs[k].copy()
                                             for k in ("rel", "w", "proj", "rel_weight")))


def oracle_batch(wl: W.Workload, h, r, t, lo, hi, seed=None, epoch=0) -> stxo.Batch:
    seed = W.negative_seed(wl) if seed is None else seed
    nh, nt = stxo.sample_negatives(h[lo:hi], r[lo:hi], t[lo:hi], wl.n_neg, wl.n_ent, seed, epoch,
                                   m_total=wl.n_triplets, global_offset=lo)
    return stxo.Batch(h[lo:hi], r[lo:hi], t[lo:hi], nh, nt)


def small_problem(model: str, dist: str, n_ent=30, n_rel=4, b=12, k=2, dim=8, rel_dim=None, seed=0,
                  margin=1.0, grid=None):
    """A tiny random problem.  With `grid`, table entries are integer multiples of 2**-grid so that
    fp32 sums of a few of them are exact (used by the finite-difference tests)."""
    rng = np.random.default_rng(seed)
    rel_dim = rel_dim or dim
    wl = W.Workload("small", 9, model, dist, n_ent, n_rel, b, dim, rel_dim, b, k, margin, 0.01, 1, 0.0, 0.0)
    h = rng.integers(0, n_ent, b).astype(np.int32)
    t = rng.integers(0, n_ent, b).astype(np.int32)
    r = rng.integers(0, n_rel, b).astype(np.int32)

    def draw(*shape, scale=1.0):
        v = rng.uniform(-scale, scale, size=shape)
        if grid is not None:
            v = np.round(v * 2.0**grid) / 2.0**grid
        return v.astype(np.float32)

    if model in ("transe", "toruse"):
        tabs = {"ent": draw(n_ent + n_rel, dim)}
        if model == "toruse":
            tabs["ent"] = np.mod(tabs["ent"], np.float32(1.0)).astype(np.float32)
    elif model == "transh":
        w = rng.standard_normal((n_rel, dim))
        w /= np.linalg.norm(w, axis=1, keepdims=True)
        if grid is not None:
            w = np.round(w * 2.0**grid) / 2.0**grid
        tabs = {"ent": draw(n_ent, dim), "rel": draw(n_rel, dim), "w": w.astype(np.float32)}
    else:
        tabs = {"ent": draw(n_ent, dim), "rel": draw(n_rel, rel_dim),
                "proj": draw(n_rel, rel_dim, dim, scale=0.5)}
    bt = oracle_batch(wl, h, r, t, 0, b, seed=77)
    return wl, tabs, bt
