"""Pins of the three parts of the oracle's backward pass that set the bar of the TransH / TransR GPU checks:
the bfloat16 operand rounding of TransR's backward products (Sec. 4.4 with the configuration's bf16
operands), the `ambiguous` flag of rows whose L1-kind subgradient sits on a jump (Sec. 4.4, 4.5), and the
comparison scales a_* that stand beside every gradient element.  No GPU needed."""
import numpy as np
import pytest
import torch

from oracle import stxo
from tests.util import oracle_config, oracle_tables, small_problem


def _rows(bt):
    hh = np.concatenate([bt.h, bt.nh]); tt = np.concatenate([bt.t, bt.nt])
    rr = np.concatenate([bt.r, np.repeat(bt.r, bt.k)])
    return hh, rr, tt


def _bf16(a):
    """Round to bfloat16 through the library's conversion, back in float64."""
    return torch.tensor(np.asarray(a, np.float32)).bfloat16().float().numpy().astype(np.float64)


# ----------------------------------------------------------------------------- (a) bf16 backward of TransR
@pytest.mark.parametrize("dist", ["l2", "l1", "l2_sq"])
@pytest.mark.parametrize("reduce", [stxo.SUM, stxo.MEAN])
def test_transr_bf16_backward_against_library_rounding(dist, reduce):
    """y = bf16(M_r) bf16(x) + r; dL/dx = bf16(M_r)^T bf16(dL/dy); dL/dM_r = bf16(dL/dy) bf16(x)^T;
    dL/dr = dL/dy unrounded: written out with numpy on operands rounded by torch.bfloat16."""
    wl, tabs, bt = small_problem("transr", dist, n_ent=25, n_rel=4, b=40, k=2, dim=8, rel_dim=6, seed=31)
    cfg = oracle_config(wl, reduce=reduce, bf16=True)
    hh, rr, tt = _rows(bt)
    x32 = tabs["ent"][hh] - tabs["ent"][tt]                                   # fp32 h - t
    xq, Mq = _bf16(x32), _bf16(tabs["proj"])
    y = np.einsum("nad,nd->na", Mq[rr], xq) + tabs["rel"].astype(np.float64)[rr]
    if dist == "l1":
        s, dd = np.abs(y).sum(1), np.sign(y)
    elif dist == "l2":
        s = np.sqrt((y * y).sum(1)); dd = y / s[:, None]
    else:
        s, dd = (y * y).sum(1), 2 * y
    b, k = bt.b, bt.k
    act = (wl.margin + np.repeat(s[:b], k) - s[b:]) > 0
    scale = 1.0 / (b * k) if reduce == stxo.MEAN else 1.0
    coef = np.zeros(b * (1 + k))
    np.add.at(coef, np.repeat(np.arange(b), k), act * scale)
    coef[b:] = -(act * scale)
    gy = dd * coef[:, None]
    gq = _bf16(gy)
    gx = np.einsum("na,nad->nd", gq, Mq[rr])
    want_ent = np.zeros((wl.n_ent, wl.dim)); np.add.at(want_ent, hh, gx); np.add.at(want_ent, tt, -gx)
    want_rel = np.zeros((wl.n_rel, wl.rel_dim)); np.add.at(want_rel, rr, gy)
    want_proj = np.zeros((wl.n_rel, wl.rel_dim, wl.dim)); np.add.at(want_proj, rr, gq[:, :, None] * xq[:, None, :])
    g = stxo.backward(cfg, oracle_tables(tabs), bt, want_gy=True)
    np.testing.assert_allclose(g.gy, gy, rtol=0, atol=1e-12)
    np.testing.assert_allclose(g.ent, want_ent, rtol=0, atol=1e-12)
    np.testing.assert_allclose(g.rel, want_rel, rtol=0, atol=1e-12)
    np.testing.assert_allclose(g.proj, want_proj, rtol=0, atol=1e-12)
    # the rounding matters at this size: the exact-input mode gives other numbers
    gx_mode = stxo.backward(oracle_config(wl, reduce=reduce, bf16=False), oracle_tables(tabs), bt)
    assert np.abs(gx_mode.proj - g.proj).max() > 1e-5 * np.abs(g.proj).max()


def test_transr_bf16_backward_is_exact_mode_on_bf16_representable_inputs():
    """Tables on a coarse grid and an L1 norm (dL/dy = 0, +-1): nothing is changed by the rounding."""
    wl, tabs, bt = small_problem("transr", "l1", n_ent=25, n_rel=4, b=40, k=1, dim=8, rel_dim=6, seed=32, grid=3)
    a = stxo.backward(oracle_config(wl, bf16=True), oracle_tables(tabs), bt)
    b = stxo.backward(oracle_config(wl, bf16=False), oracle_tables(tabs), bt)
    for name in ("ent", "rel", "proj", "ent_abs", "proj_abs"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name


# ----------------------------------------------------------------------------- (b) the ambiguous flag
def _flag(model, dist, E, rel, extra, dim):
    """One positive row (0, 0, 1) and a far negative that keeps the pair active."""
    cfg = stxo.Config(model, dist, E.shape[0], 1, dim, dim, margin=100.0, bf16_proj=False)
    tb = stxo.Tables(E, rel, **extra)
    bt = stxo.Batch([0], [0], [1], [0], [2])
    return stxo.backward(cfg, tb, bt).ambiguous


def _transh_row(y_first, dist=stxo.L1):
    # w = (0,0,0,1) is orthogonal to x, so y = x + d_r and sum|terms| of y_0 is |x_0| + |d_0| = 2
    E = np.array([[1, 0.5, 0.25, 0], [0, 0, 0, 0], [9, 9, 9, 0]], np.float32)
    d = np.array([[np.float32(-1.0) + np.float32(y_first), 0.25, 0.125, 0]], np.float32)
    w = np.array([[0, 0, 0, 1]], np.float32)
    return _flag(stxo.TRANSH, dist, E, d, dict(w=w), 4)


def _transr_row(y_first, dist=stxo.L1):
    # M = identity: y = x + r
    E = np.array([[1, 0.5, 0.25, 0.125], [0, 0, 0, 0], [9, 9, 9, 9]], np.float32)
    r = np.array([[np.float32(-1.0) + np.float32(y_first), 0.25, 0.125, 0.5]], np.float32)
    return _flag(stxo.TRANSR, dist, E, r, dict(proj=np.eye(4, dtype=np.float32)[None]), 4)


@pytest.mark.parametrize("row", [_transh_row, _transr_row])
def test_ambiguous_flag_l1(row):
    # sum|terms| of y_0 is 2: the flag is set when |y_0| <= 1e-5 * 2
    assert row(0.0)[0] == 1                      # exactly on the jump of sign()
    assert row(2e-6)[0] == 1                     # 1e-6 of the scale: an fp32 evaluation may land on either side
    assert row(-2e-6)[0] == 1
    assert row(2e-3)[0] == 0                     # 1e-3 of the scale: safely on one side
    assert row(-2e-3)[0] == 0
    assert row(1.5e-5)[0] == 1 and row(2.5e-5)[0] == 0     # the width itself: 1e-5 * 2 = 2e-5
    # the far negative row (x = (-8,...)) is never near a jump
    assert row(0.0)[1] == 0


@pytest.mark.parametrize("row", [_transh_row, _transr_row])
def test_ambiguous_flag_torus(row):
    # torus-L1 on a computed y: jumps at fractional part 0 and 1/2
    t = lambda v: row(v, stxo.TORUS_L1)[0]
    assert t(0.0) == 1 and t(1.0) == 1 and t(0.5) == 1 and t(-0.5) == 1
    assert t(0.5 + 4e-6) == 1 and t(0.5 - 4e-6) == 1 and t(4e-6) == 1
    assert t(0.25) == 0 and t(0.75) == 0 and t(0.5 + 2e-3) == 0 and t(2e-3) == 0


def test_ambiguous_flag_unused_elsewhere():
    # L2 kinds have no jump; stacked models compute y = x exactly
    assert not _transh_row(0.0, stxo.L2).any() and not _transr_row(0.0, stxo.L2_SQ).any()
    # an element of y whose terms are all zero (x_3 = d_3 = 0 and w.x = 0 in _transh_row) is 0 in any precision:
    # rows of the L1 tests above would all be flagged if it counted
    assert _transh_row(2e-3)[0] == 0
    X = np.array([[1, 0.5], [0, 0], [9, 9], [-1, 0.25]], np.float32)            # x_0 = 1 - 1 - 0 = 0 exactly
    cfg = stxo.Config(stxo.TRANSE, stxo.L1, 3, 1, 2, margin=100.0)
    assert not stxo.backward(cfg, stxo.Tables(X), stxo.Batch([0], [0], [1], [0], [2])).ambiguous.any()


# ----------------------------------------------------------------------------- (c) the comparison scales
def _plain_scales(model, tabs, bt, g, wl):
    """Sum of |separately rounded terms| with |dL/dy_j| itself as the size of dL/dy_j (no widening)."""
    hh, rr, tt = _rows(bt)
    gy = g.gy
    x = (tabs["ent"][hh] - tabs["ent"][tt]).astype(np.float64)
    out = {}
    if model == "transh":
        w = tabs["w"].astype(np.float64)[rr]
        a = (gy * w).sum(1, keepdims=True)
        s = (x * w).sum(1, keepdims=True)
        ax = np.abs(gy) + np.abs(a * w)
        out["rel"] = np.zeros_like(g.rel); np.add.at(out["rel"], rr, np.abs(gy))
        out["w"] = np.zeros_like(g.w); np.add.at(out["w"], rr, np.abs(a * x) + np.abs(s) * np.abs(gy))
    else:
        M = tabs["proj"].astype(np.float64)[rr]
        ax = np.einsum("na,nad->nd", np.abs(gy), np.abs(M))
        out["rel"] = np.zeros_like(g.rel); np.add.at(out["rel"], rr, np.abs(gy))
        out["proj"] = np.zeros_like(g.proj); np.add.at(out["proj"], rr, np.abs(gy)[:, :, None] * np.abs(x)[:, None, :])
    out["ent"] = np.zeros_like(g.ent); np.add.at(out["ent"], hh, ax); np.add.at(out["ent"], tt, ax)
    return out


# how far the widened scale may exceed the plain one: y_j is a sum of 3 (TransH) or dim + 1 (TransR) terms, and
# sum|terms| / |sum| of such a sum of random signs grows like the square root of their number
WIDEN_CAP = {"transh": 6.0, "transr": 2.0 * np.sqrt(32.0)}


@pytest.mark.parametrize("model", ["transh", "transr"])
@pytest.mark.parametrize("dist", ["l1", "l2", "l2_sq"])
@pytest.mark.parametrize("seed", [0, 1])
def test_scales_bounded_above_and_below(model, dist, seed):
    wl, tabs, bt = small_problem(model, dist, n_ent=60, n_rel=5, b=256, k=2, dim=32, rel_dim=32, seed=seed)
    cfg = oracle_config(wl, bf16=False)
    g = stxo.backward(cfg, oracle_tables(tabs), bt, want_gy=True)
    plain = _plain_scales(model, tabs, bt, g, wl)
    for name, p in plain.items():
        a = getattr(g, name + "_abs")
        val = np.abs(getattr(g, name))
        assert np.all(a >= val - 1e-12), name                                   # a scale dominates its sum
        assert np.all(a >= p * (1 - 1e-12) - 1e-15), name                         # ... and the plain scale
        if dist == "l1":                                                        # no widening for the L1 kinds
            np.testing.assert_allclose(a, p, rtol=1e-12, atol=1e-15, err_msg=name)
        else:
            assert np.all(a <= WIDEN_CAP[model] * p + 1e-15), (name, float((a / (p + 1e-300)).max()))
            assert a.sum() <= 0.75 * WIDEN_CAP[model] * p.sum(), name
        assert np.array_equal(a == 0, p == 0), name                              # the same elements are touched


def _fp32_gradients(model, dist, tabs, bt, wl):
    """The same formulas evaluated in single precision throughout (numpy float32, sums over rows in index
    order), as an fp32 kernel would: the distance to the double-precision oracle is what the scales bound."""
    f = np.float32
    hh, rr, tt = _rows(bt)
    E = tabs["ent"]
    x = E[hh] - E[tt]
    if model == "transh":
        w, d = tabs["w"][rr], tabs["rel"][rr]
        s = np.zeros(len(hh), f)
        for j in range(wl.dim):
            s = s + w[:, j] * x[:, j]
        y = (x + d) - s[:, None] * w
    else:
        M = tabs["proj"][rr]
        y = np.zeros((len(hh), wl.rel_dim), f)
        for j in range(wl.dim):
            y = y + M[:, :, j] * x[:, j:j + 1]
        y = y + tabs["rel"][rr]
    assert y.dtype == f
    sq = np.zeros(len(hh), f)
    for j in range(y.shape[1]):
        sq = sq + y[:, j] * y[:, j]
    sc = np.sqrt(sq) if dist == "l2" else sq
    b, k = bt.b, bt.k
    act = ((f(wl.margin) + np.repeat(sc[:b], k)) - sc[b:]) > 0
    coef = np.zeros(len(hh), f)
    np.add.at(coef, np.repeat(np.arange(b), k), act.astype(f))
    coef[b:] = -act.astype(f)
    gy = (coef / sc)[:, None] * y if dist == "l2" else (f(2) * coef)[:, None] * y
    out = {}
    if model == "transh":
        a = np.zeros(len(hh), f)
        for j in range(wl.dim):
            a = a + gy[:, j] * w[:, j]
        gx = gy - a[:, None] * w
        gw = -(a[:, None] * x + s[:, None] * gy)
        out["rel"] = np.zeros((wl.n_rel, wl.dim), f); np.add.at(out["rel"], rr, gy)
        out["w"] = np.zeros((wl.n_rel, wl.dim), f); np.add.at(out["w"], rr, gw)
    else:
        gx = np.zeros((len(hh), wl.dim), f)
        for a_ in range(wl.rel_dim):
            gx = gx + gy[:, a_:a_ + 1] * M[:, a_, :]
        out["rel"] = np.zeros((wl.n_rel, wl.rel_dim), f); np.add.at(out["rel"], rr, gy)
        out["proj"] = np.zeros((wl.n_rel, wl.rel_dim, wl.dim), f)
        np.add.at(out["proj"], rr, gy[:, :, None] * x[:, None, :])
    out["ent"] = np.zeros((wl.n_ent, wl.dim), f); np.add.at(out["ent"], hh, gx); np.add.at(out["ent"], tt, -gx)
    assert all(v.dtype == f for v in out.values())
    return act, out


@pytest.mark.parametrize("model", ["transh", "transr"])
@pytest.mark.parametrize("dist", ["l2", "l2_sq"])
def test_single_precision_evaluation_sits_well_inside_the_scales(model, dist):
    """|fp32 evaluation - oracle| <= 1e-5 * a_* with room to spare (the bar is not tight for honest fp32
    arithmetic), and not by orders of magnitude (the scales are not vacuous): the worst element uses between
    1/2000 and 1/4 of the bar."""
    wl, tabs, bt = small_problem(model, dist, n_ent=60, n_rel=5, b=256, k=2, dim=32, rel_dim=32, seed=3)
    cfg = oracle_config(wl, bf16=False)
    act, got = _fp32_gradients(model, dist, tabs, bt, wl)
    g = stxo.backward(cfg, oracle_tables(tabs), bt, active=act)
    for name, v in got.items():
        ref, a = getattr(g, name), getattr(g, name + "_abs")
        used = np.abs(v.astype(np.float64) - ref) / (1e-5 * a + 1e-300)
        assert used.max() <= 0.25, (name, float(used.max()))
        assert used.max() >= 5e-4, (name, float(used.max()))


# ----------------------------------------------------------------------------- the allowance of flagged rows
@pytest.mark.parametrize("model", ["transh", "transr"])
def test_allowance_of_flagged_rows_covers_any_other_branch(model):
    """tests/gpu_util.ambiguous_allowance bounds how far gradients move when flagged rows take other branches of
    an L1-kind subgradient: replace dL/dy of some rows by any vector of entries in {-1, 0, +1} * coef, push it
    through the backward formulas in numpy, and compare the movement with the bound."""
    from tests import gpu_util as G
    wl, tabs, bt = small_problem(model, "l1", n_ent=30, n_rel=4, b=48, k=2, dim=8, rel_dim=8, seed=51)
    cfg = oracle_config(wl, bf16=False)
    g = stxo.backward(cfg, oracle_tables(tabs), bt, want_gy=True)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt)
    active = fw.hinge_arg > 0
    rng = np.random.default_rng(7)
    amb = rng.random(bt.rows) < 0.1
    allow = G.ambiguous_allowance(wl, tabs, bt, active, amb, False)
    hh, rr, tt = _rows(bt)
    coef = G.pair_coefficients(active, bt.b, bt.k, False)
    gy2 = g.gy.copy()
    gy2[amb] = rng.integers(-1, 2, gy2[amb].shape) * coef[amb][:, None]
    x = (tabs["ent"][hh] - tabs["ent"][tt]).astype(np.float64)

    def grads(gy):
        out = {}
        if model == "transh":
            w = tabs["w"].astype(np.float64)[rr]
            a = (gy * w).sum(1, keepdims=True)
            s = (x * w).sum(1, keepdims=True)
            gx = gy - a * w
            out["w"] = np.zeros((wl.n_rel, wl.dim)); np.add.at(out["w"], rr, -(a * x + s * gy))
        else:
            M = tabs["proj"].astype(np.float64)[rr]
            gx = np.einsum("na,nad->nd", gy, M)
            out["proj"] = np.zeros((wl.n_rel, wl.rel_dim, wl.dim)); np.add.at(out["proj"], rr, gy[:, :, None] * x[:, None, :])
        out["rel"] = np.zeros((wl.n_rel, gy.shape[1])); np.add.at(out["rel"], rr, gy)
        out["ent"] = np.zeros((wl.n_ent, wl.dim)); np.add.at(out["ent"], hh, gx); np.add.at(out["ent"], tt, -gx)
        return out

    g1, g2 = grads(g.gy), grads(gy2)
    for name in g1:
        np.testing.assert_allclose(g1[name], getattr(g, name), rtol=0, atol=1e-12)     # the formulas are the oracle's
        moved = np.abs(g2[name] - g1[name])
        assert np.all(moved <= allow[name] + 1e-12), name
        assert moved.max() > 0.05 * allow[name].max(), name                            # ... and the bound is not idle
        assert np.all((allow[name] == 0) | (moved >= 0)), name
    # rows that are not flagged contribute nothing to the allowance
    none = G.ambiguous_allowance(wl, tabs, bt, active, np.zeros(bt.rows, bool), False)
    assert none is None
