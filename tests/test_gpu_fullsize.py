"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times: "mid" (TransE, 65,536 rows per batch) element by element, "toruse" (1,310,720 rows per batch,
4M-row table) on all scores and on sampled gradient / table rows the oracle computes one by one."""
import numpy as np
import pytest
import torch

from oracle import stxo
from paper_2502_16949_amd import binding as B
from paper_2502_16949_amd import workloads as W
from tests import gpu_util as G
from tests.util import oracle_batch, oracle_config, oracle_tables

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,which", [("mid", "first"), ("mid", "last_partial"), ("paper_transe", "first"),
                                        ("paper_toruse", "last_partial")])
def test_stacked_config_full_batch(name, which):
    """"mid", and the paper's own training shape (d = 1024, 393,216 positives per batch): every score, every
    gradient row and the whole updated table against the oracle."""
    wl = W.WORKLOADS[name]
    h, r, t = W.make_graph(wl)
    tabs = W.make_tables(wl)
    lo, hi = W.batch_slices(wl)[0 if which == "first" else -1]
    bt = oracle_batch(wl, h, r, t, lo, hi)
    cfg = oracle_config(wl)
    m = G.GpuModel(wl, tabs)
    # negatives from the GPU sampler, as in the benchmark
    hd, rd, td = G.dev_i32(h), G.dev_i32(r), G.dev_i32(t)
    nh = torch.empty(wl.batch, dtype=torch.int32, device=G.DEV)
    nt = torch.empty(wl.batch, dtype=torch.int32, device=G.DEV)
    B.stx_sample_negatives(m.ctx, hd[lo:hi], rd[lo:hi], td[lo:hi], wl.n_neg, W.negative_seed(wl), 0, wl.n_triplets,
                           lo, nh, nt)
    torch.cuda.synchronize()
    assert np.array_equal(nh[:hi - lo].cpu().numpy(), bt.nh) and np.array_equal(nt[:hi - lo].cpu().numpy(), bt.nt)
    B.stx_build_incidence(m.ctx, hd[lo:hi], rd[lo:hi], td[lo:hi], nh, nt, wl.n_neg, m.inc)
    G.check_incidence(m.incidence_numpy(), stxo.build_incidence(bt, wl.n_ent, wl.n_rel))
    m.forward()
    scores, loss = m.scores_numpy()
    fw = stxo.forward(cfg, oracle_tables(tabs), bt, want_x=False)
    G.check_scores_and_loss(scores, loss, fw, False)
    active = G.resolve_active(scores, fw, bt, wl.margin)
    g = stxo.backward(cfg, oracle_tables(tabs), bt, active=active)
    m.backward()
    cols, rows = m.grad_rows_numpy()
    G.check_grad_rows(cols, rows, g.ent, g.ent_abs, wl.dim)
    tb = oracle_tables(tabs)
    touched, _ = stxo.touched_masks(cfg, bt)
    stxo.sgd(tb.ent, g.ent, touched, wl.lr, 1 if wl.model == "toruse" else 0)
    m.sgd(wl.lr)
    torch.cuda.synchronize()
    new = m.params.ent.cpu().numpy()
    diff = np.abs(new.astype(np.float64) - tb.ent)
    if wl.model == "toruse":
        diff = np.minimum(diff, 1.0 - diff)                              # distance on the circle
        assert new.min() >= 0.0 and new.max() < 1.0
    assert np.all(diff <= G.REL_TOL * (wl.lr * g.ent_abs + np.abs(tabs["ent"]) * 2.0**-23) + 2.0**-23)
    assert np.array_equal(new[touched == 0], tabs["ent"][touched == 0])
    # the fused backward + update: same bits as the two separate calls just checked
    m2 = G.GpuModel(wl, tabs)
    B.stx_build_incidence(m2.ctx, hd[lo:hi], rd[lo:hi], td[lo:hi], nh, nt, wl.n_neg, m2.inc)
    m2.forward()
    m2.backward_sgd(wl.lr, with_grads=False)
    torch.cuda.synchronize()
    assert np.array_equal(m2.params.ent.cpu().numpy(), new)
    # the one-call step, as bench.py runs it: negatives, incidence, scores, loss and table, all the same bits
    m3 = G.GpuModel(wl, tabs)
    nh3, nt3 = torch.empty_like(nh), torch.empty_like(nt)
    batch = B.make_batch(hd[lo:hi], rd[lo:hi], td[lo:hi], wl.n_neg, W.negative_seed(wl), 0, wl.n_triplets, lo, nh3, nt3)
    B.stx_train_step(m3.ctx, batch, m3.inc, m3.params, None, wl.lr, m3.scores, m3.loss)
    torch.cuda.synchronize()
    n = (hi - lo) * wl.n_neg
    assert torch.equal(nh3[:n], nh[:n]) and torch.equal(nt3[:n], nt[:n])
    G.check_incidence(m3.incidence_numpy(), stxo.build_incidence(bt, wl.n_ent, wl.n_rel))
    s3, l3 = m3.scores_numpy()
    assert np.array_equal(s3, scores) and l3 == loss
    assert np.array_equal(m3.params.ent.cpu().numpy(), new)


def test_toruse_large_full_batch_sampled():
    wl = W.WORKLOADS["toruse"]
    h, r, t = W.make_graph(wl)
    tabs = W.make_tables(wl)
    lo, hi = W.batch_slices(wl)[0]
    bt = oracle_batch(wl, h, r, t, lo, hi)
    cfg = oracle_config(wl)
    tb = stxo.Tables(tabs["ent"])                                   # no copy of the 2 GB table
    m = G.GpuModel(wl, tabs)
    m.build(bt)
    G.check_incidence(m.incidence_numpy(), stxo.build_incidence(bt, wl.n_ent, wl.n_rel))
    m.forward()
    scores, loss = m.scores_numpy()
    fw = stxo.forward(cfg, tb, bt, want_x=False)
    G.check_scores_and_loss(scores, loss, fw, False)
    active = G.resolve_active(scores, fw, bt, wl.margin)
    m.backward()
    cols, rows = m.grad_rows_numpy()
    # sampled columns: the heaviest entity columns, every 5,000th touched column, some relation columns
    inc = stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
    seg_len = np.diff(inc.seg_ptr)
    assert np.array_equal(cols, inc.touched_cols)
    pick = set(np.argsort(seg_len)[-6:].tolist()) | set(range(0, len(cols), 5000)) | set(range(len(cols) - 5, len(cols)))
    pick = sorted(pick)
    m.sgd(wl.lr)
    torch.cuda.synchronize()
    new_rows = m.params.ent[torch.from_numpy(cols[pick].astype(np.int64)).to(G.DEV)].cpu().numpy()
    for j, s in enumerate(pick):
        want, scale = stxo.grad_column_stacked(cfg, tb, bt, active, int(cols[s]))
        err = np.abs(rows[s].astype(np.float64) - want)
        assert np.all(err <= G.REL_TOL * scale + 1e-30), (s, int(cols[s]), int(seg_len[s]), float(err.max()))
        sub = tabs["ent"][cols[s]].copy().reshape(1, -1)
        stxo.sgd(sub, want.reshape(1, -1), np.ones(1, np.uint8), wl.lr, 1)
        d = np.abs(new_rows[j].astype(np.float64) - sub[0])
        d = np.minimum(d, 1.0 - d)
        assert np.all(d <= G.REL_TOL * wl.lr * scale + 2.0**-23), (s, float(d.max()))
    # rows of the table that the batch does not touch are unchanged (spot check on a slice)
    touched = np.zeros(wl.n_ent + wl.n_rel, bool)
    touched[cols] = True
    sl = slice(1_000_000, 1_200_000)
    same = m.params.ent[sl].cpu().numpy() == tabs["ent"][sl]
    assert np.all(same[~touched[sl]])
    # the one-call step, as bench.py runs it: negatives, scores, loss and the whole 2 GB table have the same
    # bits as after the separate calls, whose results were checked against the oracle above
    ent_after = m.params.ent
    m2 = G.GpuModel(wl, tabs)
    hd, rd, td = G.dev_i32(h[lo:hi]), G.dev_i32(r[lo:hi]), G.dev_i32(t[lo:hi])
    nh2 = torch.empty((hi - lo) * wl.n_neg, dtype=torch.int32, device=G.DEV)
    nt2 = torch.empty_like(nh2)
    batch = B.make_batch(hd, rd, td, wl.n_neg, W.negative_seed(wl), 0, wl.n_triplets, lo, nh2, nt2)
    B.stx_train_step(m2.ctx, batch, m2.inc, m2.params, None, wl.lr, m2.scores, m2.loss)
    torch.cuda.synchronize()
    assert np.array_equal(nh2.cpu().numpy(), bt.nh) and np.array_equal(nt2.cpu().numpy(), bt.nt)
    s2, l2 = m2.scores_numpy()
    assert np.array_equal(s2, scores) and l2 == loss
    assert torch.equal(m2.params.ent, ent_after)
