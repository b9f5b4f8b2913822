"""End to end, on a graph whose structure a translation model can represent: training lowers the loss and link
prediction on held-out triplets rises far above chance.  The paper's accuracy figures (Hits@10 on WN18 / FB15k)
need its datasets; this is the stand-in that shows the whole path (sampler, incidence, forward, backward,
update, ranking) learns.  Oracle only (no GPU); tests/test_gpu_learns.py runs the same schedule on the GPU."""
import numpy as np
import pytest

from oracle import stxo
from paper_2502_16949_amd import workloads as W
from tests.util import oracle_config, oracle_tables

N_ENT, SHIFTS, BATCH = 200, [1, 2, 5, -3], 256
CASES = {
    # model, dist, ring, dim, lr, margin, epochs, Hits@10 both sides must reach (chance: 10 / 200 = 0.05)
    "toruse": ("toruse", "torus_l1", True, 16, 0.01, 1.0, 150, 0.85),
    "transe": ("transe", "l2", False, 16, 0.05, 1.0, 300, 0.30),
    "transh": ("transh", "l2", False, 16, 0.05, 1.0, 300, 0.30),
    "transr": ("transr", "l2", False, 32, 0.05, 1.0, 300, 0.10),   # bfloat16 projection operands; learns slowly
}


def learn_setup(name):
    model, dist, ring, dim, lr, margin, epochs, bar = CASES[name]
    train, test = W.make_shift_graph(N_ENT, SHIFTS, seed=1, ring=ring)
    wl = W.Workload("learn", 9, model, dist, N_ENT, len(SHIFTS), len(train[0]), dim, dim, BATCH, 1, margin, lr, epochs,
                    0.0, 0.0, model == "transr")
    return wl, train, test, bar


def hits_at_10(less):
    return float((1 + less <= 10).mean())


def oracle_learn(name):
    wl, (h, r, t), test, bar = learn_setup(name)
    cfg = oracle_config(wl)
    tb = oracle_tables(W.make_tables(wl))
    losses = []
    for ep in range(wl.epochs):
        total = 0.0
        for lo in range(0, len(h), wl.batch):
            hi = min(lo + wl.batch, len(h))
            nh, nt = stxo.sample_negatives(h[lo:hi], r[lo:hi], t[lo:hi], 1, wl.n_ent, W.negative_seed(wl), ep, len(h), lo)
            fw, _ = stxo.train_step(cfg, tb, stxo.Batch(h[lo:hi], r[lo:hi], t[lo:hi], nh, nt), wl.lr)
            total += fw.loss
        losses.append(total)
    hits = [hits_at_10(stxo.rank(oracle_config(wl, bf16=False), tb, *test, side)[1]) for side in (stxo.TAIL, stxo.HEAD)]
    return losses, hits, bar


@pytest.mark.parametrize("name", sorted(CASES))
def test_oracle_training_learns_the_shift_graph(name):
    wl, _, test, _ = learn_setup(name)
    start = [hits_at_10(stxo.rank(oracle_config(wl, bf16=False), oracle_tables(W.make_tables(wl)), *test, side)[1])
             for side in (stxo.TAIL, stxo.HEAD)]
    losses, hits, bar = oracle_learn(name)
    assert max(start) <= 0.15                                  # untrained tables rank at chance
    assert losses[-1] < 0.2 * losses[0]
    assert min(hits) >= bar, hits
