"""stx_train_step (one call per training step, with launches shared between independent kernels) against
the separate calls stx_sample_negatives + stx_build_incidence + stx_forward + stx_backward + stx_sgd_step.
The separate calls are checked against the oracle in the other GPU test files; the one-call step does
the same arithmetic in the same order, so every output must have the same bits.  The full-size checks
of the step against the oracle itself are in test_gpu_fullsize.py."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2502_16949_amd import binding as B
from paper_2502_16949_amd import workloads as W
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

CASES = [
    # model, dist, n_ent, n_rel, b, k, dim, rel_dim, flags
    ("transe", "l1", 1000, 20, 1000, 1, 128, 128, 0),
    ("transe", "l2", 400, 9, 777, 3, 128, 128, 0),
    ("transe", "l1", 64, 4, 2500, 2, 100, 100, 0),                # one sort pass only
    ("transe", "l2", 70000, 5, 3000, 1, 32, 32, 0),               # too many columns for the presence bitmap
    ("transe", "l2", 300, 5, 200, 1, 512, 512, 0),                # rows wider than the shared-launch forward covers
    ("toruse", "torus_l1", 1000, 20, 1024, 4, 128, 128, 0),
    ("toruse", "torus_l2", 500, 7, 600, 2, 64, 64, 0),
    ("transe", "l2", 100, 3, 50, 0, 64, 64, 0),                   # no negatives at all
    ("transe", "l2_sq", 400, 9, 777, 3, 128, 128, 0),
    ("transh", "l2_sq", 400, 9, 777, 2, 64, 64, 0),
    ("transh", "l2", 1000, 20, 1024, 1, 128, 128, B.STX_FLAG_RENORM_W),
    ("transh", "l1", 400, 9, 777, 3, 64, 64, 0),
    ("transh", "l2", 200, 5, 200, 1, 1024, 1024, 0),
    ("transr", "l2", 1000, 20, 1024, 1, 128, 128, B.STX_FLAG_BF16_PROJ),
    ("transr", "l1", 300, 40, 500, 2, 64, 32, B.STX_FLAG_BF16_PROJ),
]


@pytest.mark.parametrize("model,dist,n_ent,n_rel,b,k,dim,rel_dim,flags", CASES)
def test_train_step_equals_the_separate_calls(model, dist, n_ent, n_rel, b, k, dim, rel_dim, flags):
    """Three consecutive batches (the last one shorter), so that the alternating presence bitmaps and the
    state left by the previous step are exercised."""
    wl = W.Workload("case", 11, model, dist, n_ent, n_rel, 3 * b, dim, rel_dim, b, k, 1.0, 0.01, 1, 1.1, 1.1,
                    bool(flags & B.STX_FLAG_BF16_PROJ))
    tabs = W.make_tables(wl)
    rng = np.random.default_rng(5)
    m_total = 3 * b
    hd = G.dev_i32(rng.integers(0, n_ent, m_total))
    rd = G.dev_i32(rng.integers(0, n_rel, m_total))
    td = G.dev_i32(rng.integers(0, n_ent, m_total))
    ma, mb = G.GpuModel(wl, tabs, flags=flags), G.GpuModel(wl, tabs, flags=flags)
    nk = max(1, b * k)
    nha, nta, nhb, ntb = (torch.zeros(nk, dtype=torch.int32, device=G.DEV) for _ in range(4))
    for step, (lo, hi) in enumerate([(0, b), (b, 2 * b), (2 * b, 3 * b - 7)]):
        bb = hi - lo
        if k:
            B.stx_sample_negatives(ma.ctx, hd[lo:hi], rd[lo:hi], td[lo:hi], k, 99, 2, m_total, lo, nha, nta)
        B.stx_build_incidence(ma.ctx, hd[lo:hi], rd[lo:hi], td[lo:hi], nha if k else None, nta if k else None, k, ma.inc)
        ma.forward()
        ma.backward()
        ma.sgd(0.01)
        batch = B.make_batch(hd[lo:hi], rd[lo:hi], td[lo:hi], k, 99, 2, m_total, lo, nhb, ntb)
        # no model needs gradient storage for the one-call step: given on the first batch only
        B.stx_train_step(mb.ctx, batch, mb.inc, mb.params, mb.grads if step == 0 else None, 0.01, mb.scores, mb.loss)
        torch.cuda.synchronize()
        assert torch.equal(nha[:bb * k], nhb[:bb * k]) and torch.equal(nta[:bb * k], ntb[:bb * k])
        ia, ib = ma.incidence_numpy(), mb.incidence_numpy()
        for name in ia:
            assert np.array_equal(ia[name], ib[name]), (step, name)
        sa, la = ma.scores_numpy()
        sb, lb = mb.scores_numpy()
        assert np.array_equal(sa, sb) and la == lb, step
        for name in ("ent", "rel", "w", "proj"):
            ta, tb = getattr(ma.params, name), getattr(mb.params, name)
            assert (ta is None and tb is None) or torch.equal(ta, tb), (step, name)


def test_train_step_without_gradient_storage_for_stacked_models():
    wl = W.Workload("case", 3, "transe", "l1", 500, 10, 600, 128, 128, 600, 1, 1.0, 0.01, 1, 1.1, 1.1)
    tabs = W.make_tables(wl)
    h, r, t = W.make_graph(wl)
    hd, rd, td = G.dev_i32(h), G.dev_i32(r), G.dev_i32(t)
    m = G.GpuModel(wl, tabs)
    nh, nt = (torch.zeros(600, dtype=torch.int32, device=G.DEV) for _ in range(2))
    batch = B.make_batch(hd, rd, td, 1, 7, 0, 600, 0, nh, nt)
    before = m.params.ent.clone()
    B.stx_train_step(m.ctx, batch, m.inc, m.params, None, 0.01, m.scores, m.loss)
    torch.cuda.synchronize()
    assert not torch.equal(before, m.params.ent) and float(m.loss.item()) > 0.0
    with pytest.raises(B.StxError):                                      # the step consumed its forward pass
        m.backward()


@pytest.mark.parametrize("model,flags", [("transe", 0), ("transh", 0), ("transr", B.STX_FLAG_BF16_PROJ)])
def test_train_step_empty_batch_changes_nothing(model, flags):
    wl = W.Workload("case", 4, model, "l2", 200, 6, 100, 64, 64, 100, 1, 1.0, 0.01, 1, 0.0, 0.0, bool(flags))
    tabs = W.make_tables(wl)
    m = G.GpuModel(wl, tabs, flags=flags)
    empty = torch.zeros(0, dtype=torch.int32, device=G.DEV)
    neg = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    batch = B.make_batch(empty, empty, empty, 1, 7, 0, 100, 0, neg, neg)
    m.loss.fill_(123.0)
    B.stx_train_step(m.ctx, batch, m.inc, m.params, None, 0.01, m.scores, m.loss)
    torch.cuda.synchronize()
    assert float(m.loss.item()) == 0.0 and int(m.inc.n_touched.item()) == 0
    for name in ("ent", "rel", "w", "proj"):
        t = getattr(m.params, name)
        assert t is None or np.array_equal(t.cpu().numpy(), tabs[name])


def test_train_step_rejects_bad_arguments():
    wl = W.Workload("case", 4, "transe", "l2", 200, 6, 100, 64, 64, 100, 1, 1.0, 0.01, 1, 0.0, 0.0)
    m = G.GpuModel(wl, W.make_tables(wl))
    h = torch.zeros(101, dtype=torch.int32, device=G.DEV)           # more positives than max_batch
    neg = torch.zeros(101, dtype=torch.int32, device=G.DEV)
    scores = torch.zeros(300, dtype=torch.float32, device=G.DEV)
    with pytest.raises(B.StxError) as ei:
        B.stx_train_step(m.ctx, B.make_batch(h, h, h, 1, 7, 0, 101, 0, neg, neg), m.inc, m.params, None, 0.01,
                         scores, m.loss)
    assert ei.value.status == B.STX_ERR_BAD_ARG
    with pytest.raises(B.StxError):                                   # lr is NaN
        B.stx_train_step(m.ctx, B.make_batch(h[:10], h[:10], h[:10], 1, 7, 0, 10, 0, neg, neg), m.inc, m.params, None,
                         float("nan"), m.scores, m.loss)


LOOKAHEAD_CASES = [
    # model, dist, n_ent, n_rel, b, k, dim, flags                 what it exercises
    ("transe", "l1", 1000, 20, 1000, 1, 128, 0),                 # the benchmark's shape in small: packed dL/dx rows
    ("transe", "l2", 400, 9, 777, 3, 128, 0),                    # dense rows, several negatives
    ("toruse", "torus_l1", 1000, 20, 1024, 4, 64, 0),
    ("transh", "l2", 1000, 20, 1024, 1, 128, B.STX_FLAG_RENORM_W),   # two transposed products in the launch
    ("transe", "l1", 50, 5, 20, 1, 128, 0),                      # one sort pass, one tile: no fix-up launch to ride in
    ("transe", "l2", 3000, 5, 20, 1, 128, 0),                    # two sort passes, no fix-up launch: only k_emit runs ahead
    ("toruse", "torus_l1", 40000, 100, 5000, 2, 128, 0),         # 16 key bits, 30,000 entries: 30 sort tiles
    ("transe", "l1", 500, 10, 600, 1, 256, 0),                   # 64 lanes per row
    ("transe", "l2", 300, 6, 500, 2, 32, 0),                     # 8 lanes per row
    ("transh", "l1", 300, 6, 500, 2, 32, B.STX_FLAG_RENORM_W),
    ("transe", "l1", 20000, 50, 50000, 1, 32, 0),                # 293 sort tiles: the longest table scan in a scatter workgroup
    ("transe", "l2", 70000, 5, 3000, 1, 32, 0),                  # no presence bitmap: `next` is ignored
    ("transe", "l2", 300, 5, 200, 1, 512, 0),                    # wide rows (column slices): `next` is ignored
    ("toruse", "torus_l1", 300000, 50, 60000, 2, 32, 0),         # a large sort (540,000 entries, no bitmap): its first kernel alone
    ("transe", "l2", 200000, 30, 90000, 1, 32, 0),               # ... runs ahead, in the fix-up launch that ends the step
    ("transr", "l2", 300, 8, 500, 1, 64, B.STX_FLAG_BF16_PROJ),  # TransR: the early kernel also counts rows per relation
    ("transr", "l2", 2000, 40, 3000, 2, 128, B.STX_FLAG_BF16_PROJ),  # ... at the benchmark's width, several negatives
    ("transr", "l2", 100, 4, 700, 1, 64, B.STX_FLAG_BF16_PROJ),  # one sort pass: the early scatter pass must wait for the fix-up launch
]


@pytest.mark.parametrize("model,dist,n_ent,n_rel,b,k,dim,flags", LOOKAHEAD_CASES)
def test_train_step_with_the_next_batch_named_gives_the_same_bits(model, dist, n_ent, n_rel, b, k, dim, flags):
    """Seven steps over three batches (the last one shorter; the walk wraps around twice), once plain and once with
    every call naming the batch of the call after it, whose first build kernels then run inside this step's launches
    (from the third linked step on all three stages that can run ahead have).  After every step: same scores, loss, tables, A^T arrays; and the A arrays and
    negatives already those of the next batch.  Then a call that is given another batch than the one named."""
    wl = W.Workload("case", 12, model, dist, n_ent, n_rel, 3 * b, dim, dim, b, k, 1.0, 0.01, 1, 1.1, 1.1,
                    bool(flags & B.STX_FLAG_BF16_PROJ))
    tabs = W.make_tables(wl)
    rng = np.random.default_rng(6)
    m_total = 3 * b
    hd = G.dev_i32(rng.integers(0, n_ent, m_total))
    rd = G.dev_i32(rng.integers(0, n_rel, m_total))
    td = G.dev_i32(rng.integers(0, n_ent, m_total))
    slices = [(0, b), (b, 2 * b), (2 * b, 3 * b - 7)]
    ma, mb = G.GpuModel(wl, tabs, flags=flags), G.GpuModel(wl, tabs, flags=flags)
    nk = max(1, b * k)
    neg_a = [tuple(torch.zeros(nk, dtype=torch.int32, device=G.DEV) for _ in range(2)) for _ in slices]
    neg_b = [tuple(torch.zeros(nk, dtype=torch.int32, device=G.DEV) for _ in range(2)) for _ in slices]
    mk = lambda neg: [B.make_batch(hd[lo:hi], rd[lo:hi], td[lo:hi], k, 99, 1, m_total, lo, *neg[i])
                      for i, (lo, hi) in enumerate(slices)]
    plain, linked = mk(neg_a), B.link_batches(mk(neg_b), cyclic=True)
    for step in range(7):
        i = step % 3
        B.stx_train_step(ma.ctx, plain[i], ma.inc, ma.params, ma.grads, 0.01, ma.scores, ma.loss)
        B.stx_train_step(mb.ctx, linked[i], mb.inc, mb.params, mb.grads, 0.01, mb.scores, mb.loss)
        torch.cuda.synchronize()
        bb = slices[i][1] - slices[i][0]
        assert torch.equal(neg_a[i][0][:bb * k], neg_b[i][0][:bb * k]) and torch.equal(neg_a[i][1][:bb * k], neg_b[i][1][:bb * k])
        sa, la = ma.scores_numpy()
        sb, lb = mb.scores_numpy()
        assert np.array_equal(sa, sb) and la == lb, step
        ia, ib = ma.incidence_numpy(), mb.incidence_numpy()
        for name in ("touched_cols", "seg_ptr", "row_idx", "sign", "seg_id", "packed", "n_touched"):
            assert np.array_equal(ia[name], ib[name]), (step, name)
        for name in ("ent", "rel", "w", "proj"):
            ta, tb = getattr(ma.params, name), getattr(mb.params, name)
            assert (ta is None and tb is None) or torch.equal(ta, tb), (step, name)
    # the call after step 6 (batch 0) was announced as batch 1; give batch 2 instead: it must build from scratch
    B.stx_train_step(ma.ctx, plain[2], ma.inc, ma.params, ma.grads, 0.01, ma.scores, ma.loss)
    B.stx_train_step(mb.ctx, linked[2], mb.inc, mb.params, mb.grads, 0.01, mb.scores, mb.loss)
    # ... and then a plain build + forward on the same context (its announced batch 0 is not what comes)
    for m in (ma, mb):
        B.stx_build_incidence(m.ctx, hd[:b], rd[:b], td[:b], neg_a[0][0] if k else None, neg_a[0][1] if k else None, k, m.inc)
        m.forward()
    torch.cuda.synchronize()
    ia, ib = ma.incidence_numpy(), mb.incidence_numpy()
    for name in ia:
        assert np.array_equal(ia[name], ib[name]), name
    sa, la = ma.scores_numpy()
    sb, lb = mb.scores_numpy()
    assert np.array_equal(sa, sb) and la == lb
    for name in ("ent", "rel", "w", "proj"):
        ta, tb = getattr(ma.params, name), getattr(mb.params, name)
        assert (ta is None and tb is None) or torch.equal(ta, tb), name
    assert B.stx_check_indices(ma.ctx) == 0 and B.stx_check_indices(mb.ctx) == 0


RANDOM_CHAIN_CASES = [
    ("transe", "l1", 1000, 20, 128, 1, 0),
    ("toruse", "torus_l1", 3000, 30, 128, 2, 0),
    ("transh", "l2", 1000, 20, 128, 1, B.STX_FLAG_RENORM_W),
    ("transr", "l2", 500, 12, 64, 1, B.STX_FLAG_BF16_PROJ),
    ("transr", "l2", 100, 4, 128, 2, B.STX_FLAG_BF16_PROJ),   # one sort pass
    ("transe", "l1", 120, 3, 32, 1, 0),                        # one sort pass, 8 lanes per row
]


@pytest.mark.parametrize("model,dist,n_ent,n_rel,dim,k,flags", RANDOM_CHAIN_CASES)
def test_random_chains_of_linked_steps_give_the_same_bits(model, dist, n_ent, n_rel, dim, k, flags):
    """Eighty steps over five batches of very different sizes (1 to 1,500 positives) in random order, once plain
    and once with most calls naming a next batch: usually the one that follows, sometimes another one, sometimes
    none; now and then a separate build + forward on the same context comes in between.  Whatever stages of the
    next build ran ahead or were thrown away, every step leaves the same scores, loss, A^T arrays and tables."""
    rng = np.random.default_rng(1000 * n_ent + 10 * dim + k)
    bmax = 1500
    wl = W.Workload("case", 12, model, dist, n_ent, n_rel, 5 * bmax, dim, dim, bmax, k, 1.0, 0.01, 1, 1.1, 1.1,
                    bool(flags & B.STX_FLAG_BF16_PROJ))
    tabs = W.make_tables(wl)
    m_total = 5 * bmax
    hd = G.dev_i32(rng.integers(0, n_ent, m_total))
    rd = G.dev_i32(rng.integers(0, n_rel, m_total))
    td = G.dev_i32(rng.integers(0, n_ent, m_total))
    slices = [(q * bmax, q * bmax + s) for q, s in enumerate([bmax, 700, 1, 1499, 64])]
    ma, mb = G.GpuModel(wl, tabs, flags=flags), G.GpuModel(wl, tabs, flags=flags)
    nk = bmax * k
    neg_a = [tuple(torch.zeros(nk, dtype=torch.int32, device=G.DEV) for _ in range(2)) for _ in slices]
    neg_b = [tuple(torch.zeros(nk, dtype=torch.int32, device=G.DEV) for _ in range(2)) for _ in slices]
    mk = lambda neg: [B.make_batch(hd[lo:hi], rd[lo:hi], td[lo:hi], k, 99, 1, m_total, lo, *neg[i])
                      for i, (lo, hi) in enumerate(slices)]
    plain, linked = mk(neg_a), mk(neg_b)
    steps = 80
    order = rng.integers(0, len(slices), steps + 1)
    for s in range(steps):
        i = int(order[s])
        named = int(order[s + 1]) if rng.random() < 0.8 else int(rng.integers(0, len(slices)))
        linked[i].next = ctypes.addressof(linked[named]) if rng.random() < 0.9 else None
        B.stx_train_step(ma.ctx, plain[i], ma.inc, ma.params, ma.grads, 0.01, ma.scores, ma.loss)
        B.stx_train_step(mb.ctx, linked[i], mb.inc, mb.params, mb.grads, 0.01, mb.scores, mb.loss)
        if rng.random() < 0.1:
            lo, hi = slices[0]
            for m in (ma, mb):
                B.stx_build_incidence(m.ctx, hd[lo:hi], rd[lo:hi], td[lo:hi], neg_a[0][0], neg_a[0][1], k, m.inc)
                m.forward()
        torch.cuda.synchronize()
        sa, la = ma.scores_numpy()
        sb, lb = mb.scores_numpy()
        assert np.array_equal(sa, sb) and la == lb, s
        ia, ib = ma.incidence_numpy(), mb.incidence_numpy()
        for name in ("touched_cols", "seg_ptr", "row_idx", "sign", "seg_id", "packed", "n_touched"):
            assert np.array_equal(ia[name], ib[name]), (s, name)
        for name in ("ent", "rel", "w", "proj"):
            ta, tb = getattr(ma.params, name), getattr(mb.params, name)
            assert (ta is None and tb is None) or torch.equal(ta, tb), (s, name)
    assert B.stx_check_indices(ma.ctx) == 0 and B.stx_check_indices(mb.ctx) == 0


def test_calls_that_read_A_are_refused_while_it_holds_the_next_batch():
    """After a step that named its next batch, the A arrays of inc are the next batch's and the A^T arrays this
    batch's: stx_forward / stx_spmm / the semiring products on that inc return STX_ERR_STATE until it is built
    again; a step that did not name a batch leaves inc whole."""
    wl = W.Workload("case", 12, "transe", "l1", 1000, 20, 3000, 128, 128, 1000, 1, 1.0, 0.01, 1, 1.1, 1.1)
    tabs = W.make_tables(wl)
    h, r, t = W.make_graph(wl)
    hd, rd, td = G.dev_i32(h), G.dev_i32(r), G.dev_i32(t)
    m = G.GpuModel(wl, tabs)
    neg = [tuple(torch.zeros(1000, dtype=torch.int32, device=G.DEV) for _ in range(2)) for _ in range(3)]
    bts = B.link_batches([B.make_batch(hd[lo:lo + 1000], rd[lo:lo + 1000], td[lo:lo + 1000], 1, 5, 0, 3000, lo, *neg[i])
                          for i, lo in enumerate((0, 1000, 2000))])
    out = torch.empty(2000, 128, dtype=torch.float32, device=G.DEV)
    B.stx_train_step(m.ctx, bts[0], m.inc, m.params, None, 0.01, m.scores, m.loss)
    for call in (lambda: m.forward(), lambda: B.stx_spmm(m.ctx, m.inc, m.params, out),
                 lambda: B.stx_spmm_semiring(m.ctx, m.inc, m.params, B.STX_DISTMULT, out)):
        with pytest.raises(B.StxError) as e:
            call()
        assert e.value.status == B.STX_ERR_STATE
    B.stx_train_step(m.ctx, bts[1], m.inc, m.params, None, 0.01, m.scores, m.loss)
    B.stx_train_step(m.ctx, bts[2], m.inc, m.params, None, 0.01, m.scores, m.loss)   # names no batch
    B.stx_spmm(m.ctx, m.inc, m.params, out)
    m.forward()
    torch.cuda.synchronize()
    want = (tabs_after := m.params.ent.cpu().numpy())
    hh = np.concatenate([h[2000:], neg[2][0].cpu().numpy()]); tt = np.concatenate([t[2000:], neg[2][1].cpu().numpy()])
    rr = np.concatenate([r[2000:], r[2000:]])
    x = (want[hh] + want[wl.n_ent + rr]) - want[tt]
    assert np.array_equal(out.cpu().numpy(), x)
