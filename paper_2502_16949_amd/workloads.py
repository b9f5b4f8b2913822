"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws inputs (graphs and initial tables) with numpy.  It holds none of the
method's arithmetic and imports neither the HIP binding nor the CPU oracle, so both sides can be
fed the same arrays.

The graphs stand in for the public knowledge graphs the paper trains on (its dataset table:
FB15k 14,951 entities / 1,345 relations / 483,142 triplets; FB15k-237 14,541 / 237 / 272,115),
which are not available here: shapes come from that table, degree laws are Zipf as stated below.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    index: int           # 1-based position in the configuration list; seeds derive from it
    model: str           # "transe" | "transh" | "transr" | "toruse"
    dist: str            # "l1" | "l2" | "torus_l1" | "torus_l2"
    n_ent: int
    n_rel: int
    n_triplets: int
    dim: int
    rel_dim: int
    batch: int
    n_neg: int
    margin: float
    lr: float
    epochs: int
    zipf_ent: float      # 0 => uniform
    zipf_rel: float      # 0 => uniform
    bf16_proj: bool = False

    @property
    def rows_per_batch(self) -> int:
        return self.batch * (1 + self.n_neg)

    @property
    def n_batches(self) -> int:
        return -(-self.n_triplets // self.batch)

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "tiny": Workload("tiny", 1, "transe", "l2", 1_000, 20, 10_000, 32, 32, 1_024, 1, 1.0, 0.01, 5, 0.0, 0.0),
    "mid": Workload("mid", 2, "transe", "l1", 15_000, 1_350, 480_000, 128, 128, 32_768, 1, 1.0, 0.01, 20,
                    1.1, 1.3),
    "transh": Workload("transh", 3, "transh", "l2", 15_000, 1_350, 480_000, 128, 128, 32_768, 1, 1.0, 0.01,
                       20, 1.1, 1.3),
    # no learning rate is given for this configuration; 0.01 with a summed loss diverges within an epoch
    # (M_r receives thousands of rank-one terms per step), so the paper's own 0.0004 (Sec. 5.3) is used
    "transr": Workload("transr", 4, "transr", "l2", 14_500, 237, 272_000, 128, 128, 16_384, 1, 1.0, 0.0004,
                       20, 1.1, 1.3, True),
    "toruse": Workload("toruse", 5, "toruse", "torus_l1", 4_000_000, 1_000, 20_000_000, 128, 128, 262_144,
                       4, 1.0, 0.01, 1, 1.05, 1.2),
    # The paper's own training shapes (Sec. 5.3: embedding 1024 and batch 12 x 32,768 for TransE / TorusE, 128 and
    # 2 x 32,768 for TransR; L2 or L2-torus dissimilarity, margin 0.5, learning rate 0.0004, one pre-generated
    # negative per positive) on a graph with the sizes of FB15k's training split (Table 3).
    "paper_transe": Workload("paper_transe", 6, "transe", "l2", 14_951, 1_345, 483_142, 1_024, 1_024, 393_216, 1,
                             0.5, 0.0004, 1, 1.1, 1.3),
    "paper_toruse": Workload("paper_toruse", 7, "toruse", "torus_l2", 14_951, 1_345, 483_142, 1_024, 1_024, 393_216,
                             1, 0.5, 0.0004, 1, 1.1, 1.3),
    "paper_transr": Workload("paper_transr", 8, "transr", "l2", 14_951, 1_345, 483_142, 128, 128, 65_536, 1, 0.5,
                             0.0004, 1, 1.1, 1.3, True),
}


def _zipf_draw(rng: np.random.Generator, n_items: int, s: float, size: int, perm: np.ndarray | None):
    """size draws with P(rank j) proportional to j**-s (j = 1..n_items); s == 0 is uniform.
    Ranks are mapped to ids through `perm` (a permutation of 0..n_items-1) when given."""
    if s == 0.0:
        ids = rng.integers(0, n_items, size=size, dtype=np.int64)
    else:
        w = np.arange(1, n_items + 1, dtype=np.float64) ** (-s)
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        u = rng.random(size)
        ids = np.searchsorted(cdf, u, side="right")
        np.minimum(ids, n_items - 1, out=ids)
    if perm is not None:
        ids = perm[ids]
    return ids.astype(np.int32)


def make_graph(wl: Workload):
    """(h, r, t) int32 arrays of length n_triplets.  Heads and tails are drawn independently
    (self-loops and duplicate triplets are allowed).  Seed = 1000 + index."""
    rng = np.random.Generator(np.random.PCG64(1000 + wl.index))
    perm_e = rng.permutation(wl.n_ent) if wl.zipf_ent else None
    perm_r = rng.permutation(wl.n_rel) if wl.zipf_rel else None
    h = _zipf_draw(rng, wl.n_ent, wl.zipf_ent, wl.n_triplets, perm_e)
    t = _zipf_draw(rng, wl.n_ent, wl.zipf_ent, wl.n_triplets, perm_e)
    r = _zipf_draw(rng, wl.n_rel, wl.zipf_rel, wl.n_triplets, perm_r)
    return h, r, t


# Test triplets for link prediction: 59,071 is the size of FB15k's test split (the paper's dataset table).
N_TEST_FB15K = 59_071


def make_test_triplets(wl: Workload, n: int = N_TEST_FB15K):
    """(h, r, t) of n held-out triplets drawn from the same degree laws and id permutations as the training
    graph, with their own seed (4000 + index)."""
    rng0 = np.random.Generator(np.random.PCG64(1000 + wl.index))          # the graph's permutations, redrawn
    perm_e = rng0.permutation(wl.n_ent) if wl.zipf_ent else None
    perm_r = rng0.permutation(wl.n_rel) if wl.zipf_rel else None
    rng = np.random.Generator(np.random.PCG64(4000 + wl.index))
    h = _zipf_draw(rng, wl.n_ent, wl.zipf_ent, n, perm_e)
    t = _zipf_draw(rng, wl.n_ent, wl.zipf_ent, n, perm_e)
    r = _zipf_draw(rng, wl.n_rel, wl.zipf_rel, n, perm_r)
    return h, r, t


def make_shift_graph(n_ent: int, shifts, seed: int, ring: bool, test_share: float = 0.1):
    """A graph with structure a translation model can learn: entities are the positions 0..n_ent-1 of a line
    (or of a ring), relation i joins every position h to h + shifts[i] where that exists (modulo n_ent on the
    ring).  Returns ((h, r, t) for training, (h, r, t) held out), shuffled with the given seed."""
    hs, rs, ts = [], [], []
    for ri, sft in enumerate(shifts):
        for hh in range(n_ent):
            tt = (hh + sft) % n_ent if ring else hh + sft
            if 0 <= tt < n_ent:
                hs.append(hh); rs.append(ri); ts.append(tt)
    h, r, t = (np.array(a, np.int32) for a in (hs, rs, ts))
    p = np.random.Generator(np.random.PCG64(seed)).permutation(len(h))
    h, r, t = h[p], r[p], t[p]
    n_test = int(len(h) * test_share)
    return (h[n_test:], r[n_test:], t[n_test:]), (h[:n_test], r[:n_test], t[:n_test])


def make_tables(wl: Workload):
    """Initial parameter tables as a dict of fp32 arrays.  Seed = 2000 + index.

    transe / toruse: {"ent": X = [E;R], (n_ent+n_rel) x dim}, uniform in (-6/sqrt(dim), 6/sqrt(dim));
                     for toruse the draw is then reduced modulo 1 into [0, 1).
    transh: {"ent": E, "rel": d_r, "w": w_r}, w_r rows of unit Euclidean length.
    transr: {"ent": E, "rel": r (n_rel x rel_dim), "proj": M_r (n_rel x rel_dim x dim)} with
            M_r entries normal with variance 1/dim."""
    rng = np.random.Generator(np.random.PCG64(2000 + wl.index))
    a = 6.0 / np.sqrt(wl.dim)

    def uni(rows, cols, bound=a):
        out = np.empty((rows, cols), np.float32)
        step = max(1, (1 << 22) // cols)
        for i in range(0, rows, step):  # chunked so the 4M-row table never needs a float64 copy
            out[i:i + step] = rng.uniform(-bound, bound, size=(min(step, rows - i), cols))
        return out

    if wl.model in ("transe", "toruse"):
        x = uni(wl.n_ent + wl.n_rel, wl.dim)
        if wl.model == "toruse":
            np.mod(x, np.float32(1.0), out=x)
            x[x >= 1.0] = 0.0
        return {"ent": x}
    if wl.model == "transh":
        e = uni(wl.n_ent, wl.dim)
        d_r = uni(wl.n_rel, wl.dim)
        w = rng.standard_normal((wl.n_rel, wl.dim))
        w /= np.linalg.norm(w, axis=1, keepdims=True)
        return {"ent": e, "rel": d_r, "w": w.astype(np.float32)}
    if wl.model == "transr":
        e = uni(wl.n_ent, wl.dim)
        r = uni(wl.n_rel, wl.rel_dim, 6.0 / np.sqrt(wl.rel_dim))
        m = rng.standard_normal((wl.n_rel, wl.rel_dim, wl.dim)) * np.sqrt(1.0 / wl.dim)
        return {"ent": e, "rel": r, "proj": m.astype(np.float32)}
    raise ValueError(wl.model)


def negative_seed(wl: Workload) -> int:
    return 3000 + wl.index


def batch_slices(wl: Workload):
    """Contiguous batches in stored order, no shuffling, last partial batch kept."""
    return [(s, min(s + wl.batch, wl.n_triplets)) for s in range(0, wl.n_triplets, wl.batch)]
