"""GPU parity for the TransR step (per-relation projection on the matrix cores, bfloat16 operands and
fp32 accumulation) against the oracle in its bfloat16-emulating mode and in its exact-input mode."""
import numpy as np
import pytest
import torch

from oracle import stxo
from paper_2502_16949_amd import binding as B
from paper_2502_16949_amd import workloads as W
from tests import gpu_util as G
from tests.util import oracle_batch, oracle_config, oracle_tables

pytestmark = pytest.mark.gpu

BF16_TOL = 1e-2          # bar for quantities that pass through a bfloat16 rounding of a computed value


BULK_TOL, BULK_FRAC = 1e-5, 0.998   # share of the elements of dE / dM that must meet the fp32 bar itself (measured: 0.9990 - 1)
MAX_AMBIGUOUS_ROWS = 0.02          # largest share of a batch's rows that may sit on a jump of an L1-kind subgradient


def _bulk_and_bar(got, ref, scale, what, allowance=None):
    """Elementwise: everything within BF16_TOL * scale (a computed dL/dy that lands on the other side
    of a bfloat16 rounding boundary moves one product by 2^-8 of itself), with headroom, and nearly everything
    within the fp32 bar.  allowance: see G.ambiguous_allowance."""
    extra = np.zeros_like(ref) if allowance is None else allowance
    err = np.abs(got.astype(np.float64) - ref)
    assert np.all(err <= BF16_TOL * scale + extra + 1e-30), (what, float((err / (scale + 1e-30)).max()))
    tight = extra == 0
    used = float((err[tight] / (BF16_TOL * scale[tight] + 1e-30)).max()) if tight.any() else 0.0
    G.USAGE.append((what + " (1e-2 bar)", used))
    assert used <= G.HEADROOM, (what, used)
    ok = err[tight] <= BULK_TOL * scale[tight] + 1e-30
    G.USAGE.append((what + " (share within 1e-5)", float(ok.mean()) if ok.size else 1.0))
    assert ok.size == 0 or ok.mean() >= BULK_FRAC, (what, float(ok.mean()))


def check_transr_step(wl, tabs, bt, reduce, lr=0.01):
    cfg_b = oracle_config(wl, reduce=reduce, bf16=True)
    cfg_x = oracle_config(wl, reduce=reduce, bf16=False)
    m = G.GpuModel(wl, tabs, reduce=reduce, flags=B.STX_FLAG_BF16_PROJ)
    m.build(bt)
    m.forward()
    scores, loss = m.scores_numpy()
    fw = stxo.forward(cfg_b, oracle_tables(tabs), bt, want_x=False)
    G.check_scores_and_loss(scores, loss, fw, reduce == B.STX_MEAN)           # 1e-5 against the same roundings
    fx = stxo.forward(cfg_x, oracle_tables(tabs), bt, want_x=False)
    np.testing.assert_allclose(scores, fx.scores, rtol=BF16_TOL)              # 1e-2 against exact inputs
    active = G.resolve_active(scores, fw, bt, wl.margin)
    g = stxo.backward(cfg_b, oracle_tables(tabs), bt, active=active)
    m.backward()
    torch.cuda.synchronize()
    u = int(m.inc.n_touched.item())
    cols = m.inc.at_touched_cols[:u].cpu().numpy()
    rows = m.grads.rows[:u].cpu().numpy()
    is_ent = cols < wl.n_ent
    ec, rc = cols[is_ent], cols[~is_ent] - wl.n_ent
    # rows whose L1-kind subgradient sits on a jump: the elements they feed get G.ambiguous_allowance on top of
    # their bar, nothing is left out of the comparison
    amb = g.ambiguous.astype(bool)                                           # only L1 kinds can set it
    assert amb.mean() <= MAX_AMBIGUOUS_ROWS, amb.mean()
    allow = G.ambiguous_allowance(wl, tabs, bt, active, amb, reduce == B.STX_MEAN, bf16=True) or \
        {"ent": None, "rel": None, "proj": None}
    pick = lambda a, sel: None if a is None else a[sel]
    _bulk_and_bar(rows[is_ent][:, :wl.dim], g.ent[ec], g.ent_abs[ec], "transr dE", pick(allow["ent"], ec))
    # dL/dr is a plain fp32 sum of dL/dy: the fp32 bar applies
    G.check_grad_rows(rc, rows[~is_ent], g.rel, g.rel_abs, wl.rel_dim, what="transr dr", allowance=allow["rel"])
    proj = m.grads.proj.cpu().numpy()
    _bulk_and_bar(proj[rc], g.proj[rc], g.proj_abs[rc], "transr dM", pick(allow["proj"], rc))
    # relations absent from the batch got no gradient in the oracle either
    absent = np.ones(wl.n_rel, bool); absent[rc] = False
    assert not np.any(g.proj_abs[absent])
    # update
    tb = oracle_tables(tabs)
    m_ent, m_rel = stxo.touched_masks(cfg_b, bt)
    stxo.sgd(tb.ent, g.ent, m_ent, lr, 0)
    stxo.sgd(tb.rel, g.rel, m_rel, lr, 0)
    stxo.sgd(tb.proj, g.proj, m_rel, lr, 0)
    m.sgd(lr)
    torch.cuda.synchronize()
    for name, new, ref, old, gabs, mask in (
            ("ent", m.params.ent, tb.ent, tabs["ent"], g.ent_abs, m_ent),
            ("rel", m.params.rel, tb.rel, tabs["rel"], g.rel_abs, m_rel),
            ("proj", m.params.proj, tb.proj, tabs["proj"], g.proj_abs, m_rel)):
        new = new.cpu().numpy()
        assert np.array_equal(new[mask == 0], old[mask == 0]), name
        diff = np.abs(new.astype(np.float64) - ref)
        tol = G.REL_TOL if name == "rel" else BF16_TOL
        extra = 0.0 if allow[name] is None else lr * allow[name]
        assert np.all(diff <= tol * lr * gabs + np.abs(old) * 2.0**-22 + 2.0**-23 + extra), (name, diff.max())


CASES = [
    # dist, n_ent, n_rel, b, k, dim, rel_dim, zipf
    ("l2", 1000, 20, 1024, 1, 128, 128, 1.1),
    ("l2", 400, 40, 900, 2, 128, 128, 1.3),       # many small relations: chunks spanning several of them
    ("l1", 300, 3, 777, 1, 128, 128, 0.0),        # three large relations: runs crossing many chunks
    ("l2", 300, 5, 300, 1, 64, 32, 0.0),
    ("l2", 300, 5, 333, 2, 32, 64, 0.0),
    ("l2", 200, 7, 500, 1, 256, 128, 1.1),
    ("l1", 200, 7, 260, 1, 128, 256, 1.1),
    ("l2", 150, 4, 200, 1, 256, 256, 0.0),        # four 128 x 128 blocks of dL/dM_r
    ("l2", 150, 6, 130, 1, 96, 160, 0.0),         # tile counts that are not powers of two
    ("l2", 50, 1, 40, 1, 32, 32, 0.0),            # one relation, one partly filled item
    ("l2", 500, 300, 100, 1, 64, 64, 0.0),        # more relations than rows: every item nearly empty
    ("l2_sq", 400, 40, 900, 2, 128, 128, 1.3),
    # whole positives with their negatives per 64-slot tile (1 + k divides 64): the kernel that runs projection,
    # distances, hinge and the first backward product together
    ("l2", 400, 40, 700, 3, 128, 128, 1.3),       # 16 positives and their 48 negatives per item
    ("l1", 300, 9, 333, 7, 64, 96, 1.1),          # 8 + 56
    ("torus_l2", 200, 5, 50, 31, 32, 32, 0.0),    # 2 + 62
    ("l2", 200, 5, 40, 63, 64, 64, 0.0),          # 1 + 63
    ("l2", 300, 6, 500, 4, 128, 128, 1.1),        # 5 does not divide 64: the separate kernels
]


@pytest.mark.parametrize("reduce", [B.STX_SUM, B.STX_MEAN])
@pytest.mark.parametrize("dist,n_ent,n_rel,b,k,dim,rel_dim,zipf", CASES)
def test_transr_step_matches_oracle(dist, n_ent, n_rel, b, k, dim, rel_dim, zipf, reduce):
    wl = W.Workload("case", 7, "transr", dist, n_ent, n_rel, b, dim, rel_dim, b, k, 1.0, 0.01, 1, zipf, zipf, True)
    seed = dim + b
    h, r, t = W.make_graph(wl.scaled(index=seed))
    tabs = W.make_tables(wl.scaled(index=seed))
    bt = oracle_batch(wl, h, r, t, 0, b, seed=seed)
    check_transr_step(wl, tabs, bt, reduce)


def test_transr_without_negatives():
    """k = 0: scores of the positives, zero loss, no pair is active, so every gradient is zero and no table moves."""
    wl = W.Workload("case", 7, "transr", "l2", 300, 6, 500, 128, 128, 500, 0, 1.0, 0.01, 1, 1.1, 1.1, True)
    h, r, t = W.make_graph(wl)
    tabs = W.make_tables(wl)
    check_transr_step(wl, tabs, oracle_batch(wl, h, r, t, 0, 500), B.STX_SUM)


@pytest.mark.parametrize("name,which", [("transr", "first"), ("transr", "last_partial"), ("paper_transr", "first")])
def test_transr_config_full_batch(name, which):
    wl = W.WORKLOADS[name]
    h, r, t = W.make_graph(wl)
    tabs = W.make_tables(wl)
    lo, hi = W.batch_slices(wl)[0 if which == "first" else -1]
    check_transr_step(wl, tabs, oracle_batch(wl, h, r, t, lo, hi), B.STX_SUM, lr=wl.lr)


def test_transr_identity_projection_is_transe():
    """M_r = I (exact in bfloat16): scores equal TransE's on [E; r] up to the rounding of h - t."""
    wl = W.Workload("case", 7, "transr", "l2", 300, 6, 512, 128, 128, 512, 1, 1.0, 0.01, 1, 0.0, 0.0, True)
    h, r, t = W.make_graph(wl)
    tabs = W.make_tables(wl)
    tabs["proj"] = np.tile(np.eye(128, dtype=np.float32), (6, 1, 1))
    bt = oracle_batch(wl, h, r, t, 0, 512)
    mr = G.GpuModel(wl, tabs, flags=B.STX_FLAG_BF16_PROJ)
    mr.build(bt); mr.forward()
    me = G.GpuModel(wl.scaled(model="transe"), {"ent": np.concatenate([tabs["ent"], tabs["rel"]])})
    me.build(bt); me.forward()
    sr, _ = mr.scores_numpy()
    se, _ = me.scores_numpy()
    np.testing.assert_allclose(sr, se, rtol=5e-3)                          # h - t is rounded to bfloat16


def test_transr_needs_the_bf16_flag_and_32_wide_dims():
    for kw in (dict(flags=0), dict(dim=48, flags=B.STX_FLAG_BF16_PROJ), dict(rel_dim=288, flags=B.STX_FLAG_BF16_PROJ)):
        base = dict(model="transr", dist="l2", n_ent=100, n_rel=5, dim=64, max_batch=64, max_neg=1, rel_dim=64)
        base.update(kw)
        with pytest.raises(B.StxError) as ei:
            B.stx_workspace_bytes(B.make_config(**base))
        assert ei.value.status == B.STX_ERR_UNSUPPORTED
