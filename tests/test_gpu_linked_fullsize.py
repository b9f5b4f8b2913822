"""The path bench.py times, at its full sizes: chains of stx_train_step calls in which every call names the batch
of the call after it (so that the first kernels of the next build run inside this step's launches), on "mid",
"transh", "transr" and "paper_transr" (1,345 relations: several planner workgroups), walking through the short last batch of the epoch and back to its first batches.
After every step the linked chain must leave the same bits as the plain chain (negatives, scores, loss, A^T
arrays, every table); the first two steps are also compared with the oracle advancing its own tables."""
import numpy as np
import pytest
import torch

from oracle import stxo
from paper_2502_16949_amd import binding as B
from paper_2502_16949_amd import workloads as W
from tests import gpu_util as G
from tests.util import oracle_batch, oracle_config, oracle_tables

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["mid", "transh", "transr", "paper_transr"])
def test_linked_steps_at_full_size(name):
    wl = W.WORKLOADS[name]
    h, r, t = W.make_graph(wl)
    tabs = W.make_tables(wl)
    slices = W.batch_slices(wl)
    assert slices[-1][1] - slices[-1][0] < wl.batch                    # the epoch ends with a short batch
    n = len(slices)
    walk = [n - 3, n - 2, n - 1, 0, 1, 2]                               # ... which the walk passes through
    flags = {"transh": B.STX_FLAG_RENORM_W, "transr": B.STX_FLAG_BF16_PROJ}.get(wl.model, 0)
    ma, mb = G.GpuModel(wl, tabs, flags=flags), G.GpuModel(wl, tabs, flags=flags)
    hd, rd, td = G.dev_i32(h), G.dev_i32(r), G.dev_i32(t)
    nk = wl.batch * wl.n_neg
    neg = lambda: [tuple(torch.zeros(nk, dtype=torch.int32, device=G.DEV) for _ in range(2)) for _ in walk]
    neg_a, neg_b = neg(), neg()
    mk = lambda ng: [B.make_batch(hd[lo:hi], rd[lo:hi], td[lo:hi], wl.n_neg, W.negative_seed(wl), 0, wl.n_triplets,
                                  lo, *ng[j]) for j, (lo, hi) in enumerate(slices[i] for i in walk)]
    plain, linked = mk(neg_a), B.link_batches(mk(neg_b))
    cfg = oracle_config(wl)
    tb = oracle_tables(tabs)
    for step, i in enumerate(walk):
        lo, hi = slices[i]
        B.stx_train_step(ma.ctx, plain[step], ma.inc, ma.params, None, wl.lr, ma.scores, ma.loss)
        B.stx_train_step(mb.ctx, linked[step], mb.inc, mb.params, None, wl.lr, mb.scores, mb.loss)
        torch.cuda.synchronize()
        bk = (hi - lo) * wl.n_neg
        assert torch.equal(neg_a[step][0][:bk], neg_b[step][0][:bk]) and torch.equal(neg_a[step][1][:bk], neg_b[step][1][:bk])
        sa, la = ma.scores_numpy()
        sb, lb = mb.scores_numpy()
        assert np.array_equal(sa, sb) and la == lb, step
        ia, ib = ma.incidence_numpy(), mb.incidence_numpy()
        for key in ("touched_cols", "seg_ptr", "row_idx", "sign", "seg_id", "packed", "n_touched"):
            assert np.array_equal(ia[key], ib[key]), (step, key)
        for key in ("ent", "rel", "w", "proj"):
            ta, tb_ = getattr(ma.params, key), getattr(mb.params, key)
            assert (ta is None and tb_ is None) or torch.equal(ta, tb_), (step, key)
        if step < 2:       # the oracle's own trajectory: every score, the loss, every table
            bt = oracle_batch(wl, h, r, t, lo, hi)
            assert np.array_equal(neg_b[step][0][:bk].cpu().numpy(), bt.nh)
            assert np.array_equal(neg_b[step][1][:bk].cpu().numpy(), bt.nt)
            G.check_incidence(ib, stxo.build_incidence(bt, wl.n_ent, wl.n_rel), transpose_only=True)
            fw, _ = stxo.train_step(cfg, tb, bt, wl.lr, renorm_w=True)
            # the tables entering step 1 already differ by the rounding of step 0; where TransR rounds operands
            # computed from them to bfloat16, a few land on the other side of a rounding boundary and the score
            # moves by up to 2^-8 of one product: the bar stated for bfloat16 inputs, and nearly all at the fp32 one
            if step == 0 or wl.model != "transr":
                np.testing.assert_allclose(sb, fw.scores, rtol=1e-5 if step == 0 else 3e-5)
            else:
                np.testing.assert_allclose(sb, fw.scores, rtol=1e-2)
                # (measured 0.9995 at "transr", 0.9968 at "paper_transr", whose first step moves four times the rows)
                assert np.mean(np.abs(sb - fw.scores) <= 3e-5 * fw.scores) >= (0.999 if name == "transr" else 0.995)
            assert abs(lb - fw.loss) <= 1e-4 * fw.loss
            for key in ("ent", "rel", "w", "proj"):
                ref = getattr(tb, key)
                if ref is not None:
                    got = getattr(mb.params, key).cpu().numpy()
                    bar = 2e-5 if not (key in ("ent", "proj") and wl.model == "transr") else 2e-4   # bf16 operands
                    assert np.abs(got.astype(np.float64) - ref).max() <= bar, (step, key)
    assert B.stx_check_indices(ma.ctx) == 0 and B.stx_check_indices(mb.ctx) == 0
