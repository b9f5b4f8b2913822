"""Pins of the oracle's floating-point side: distances, loss, the four models, gradients, SGD.
Hand-computed values, closed forms, reductions between models, finite differences and a
library autograd run over plain index_select.  No GPU needed."""
import numpy as np
import pytest
import torch

from oracle import stxo
from tests.util import DIST, MODEL, oracle_config, oracle_tables, small_problem

E0 = np.empty(0, np.int32)


def _one(h, r, t, nh=E0, nt=E0):
    return stxo.Batch([h], [r], [t], nh, nt)


# ----------------------------------------------------------------------------- distances
def test_hand_computed_distances():
    # X = [E;R] with 3 entities and 1 relation, dim 2: h=(3,0), t=(0,0), r=(0,-4) -> y=(3,-4)
    X = np.array([[3, 0], [0, 0], [9, 9], [0, -4]], np.float32)
    for dist, want in ((stxo.L1, 7.0), (stxo.L2, 5.0), (stxo.L2_SQ, 25.0)):     # the last: TransC's row of Table 2
        cfg = stxo.Config(stxo.TRANSE, dist, 3, 1, 2)
        fw = stxo.forward(cfg, stxo.Tables(X), _one(0, 0, 1))
        assert fw.scores[0] == want and np.array_equal(fw.x[0], [3, -4])


def test_hand_computed_relation_weight():
    # the TransM row of Table 2: the same y = (3,-4) with relation weight 2
    X = np.array([[3, 0], [0, 0], [9, 9], [0, -4]], np.float32)
    for dist, want in ((stxo.L1, 14.0), (stxo.L2, 10.0), (stxo.L2_SQ, 50.0)):
        cfg = stxo.Config(stxo.TRANSE, dist, 3, 1, 2)
        fw = stxo.forward(cfg, stxo.Tables(X, rel_weight=np.array([2.0], np.float32)), _one(0, 0, 1))
        assert fw.scores[0] == want


def test_hand_computed_torus():
    # y = (0.25, 0.75, 0.5, 0, -0.25, 1.25): min(f,1-f) = .25 .25 .5 0 .25 .25
    y = np.array([0.25, 0.75, 0.5, 0.0, -0.25, 1.25], np.float32)
    X = np.stack([y, np.zeros(6, np.float32), np.zeros(6, np.float32)])          # h=y, t=0, r=0
    cfg = stxo.Config(stxo.TORUSE, stxo.TORUS_L1, 2, 1, 6)
    assert stxo.forward(cfg, stxo.Tables(X), _one(0, 0, 1)).scores[0] == 1.5
    cfg2 = stxo.Config(stxo.TORUSE, stxo.TORUS_L2, 2, 1, 6)
    assert stxo.forward(cfg2, stxo.Tables(X), _one(0, 0, 1)).scores[0] == pytest.approx(np.sqrt(0.5), abs=1e-15)  # 4*(1/16) + 1/4


def test_torus_equals_l1_for_small_entries():
    rng = np.random.default_rng(0)
    X = rng.uniform(-0.15, 0.15, (12, 8)).astype(np.float32)                    # |h+r-t| < 1/2
    bt = stxo.Batch([0, 1, 2], [0, 1, 0], [3, 4, 5], [6, 1, 2], [3, 7, 5])
    a = stxo.forward(stxo.Config(stxo.TORUSE, stxo.TORUS_L1, 10, 2, 8), stxo.Tables(X), bt)
    b = stxo.forward(stxo.Config(stxo.TRANSE, stxo.L1, 10, 2, 8), stxo.Tables(X), bt)
    np.testing.assert_allclose(a.scores, b.scores, rtol=0, atol=1e-6)            # f=1+y rounds in fp32
    assert a.loss == pytest.approx(b.loss, abs=1e-5)


# ----------------------------------------------------------------------------- loss
def test_loss_negative_equal_to_positive_gives_margin_and_zero_gradient():
    wl, tabs, bt = small_problem("transe", "l2", b=5, k=1, seed=2, margin=0.75)
    bt = stxo.Batch(bt.h, bt.r, bt.t, bt.h, bt.t)                                # negatives = positives
    cfg = oracle_config(wl)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt)
    np.testing.assert_allclose(fw.hinge_arg, 0.75, rtol=0, atol=1e-14)                # (m + d) - d in double
    assert fw.loss == pytest.approx(5 * 0.75, abs=1e-13)
    g = stxo.backward(cfg, oracle_tables(tabs), bt)
    assert np.all(np.abs(g.ent) <= 1e-14) and np.any(g.ent_abs > 0.1)             # terms cancel pairwise
    cfg_m = oracle_config(wl, reduce=stxo.MEAN)
    assert stxo.forward(cfg_m, oracle_tables(tabs), bt).loss == pytest.approx(0.75)


def test_loss_zero_margin_far_negative():
    X = np.array([[0, 0], [1, 0], [50, 0], [0, 0]], np.float32)                  # 3 entities + 1 relation
    cfg = stxo.Config(stxo.TRANSE, stxo.L2, 3, 1, 2, margin=0.0)
    fw = stxo.forward(cfg, stxo.Tables(X), _one(0, 0, 1, [0], [2]))              # d+=1, d-=50
    assert fw.loss == 0.0 and fw.hinge_arg[0] == -49.0
    g = stxo.backward(cfg, stxo.Tables(X), _one(0, 0, 1, [0], [2]))
    assert np.all(g.ent == 0) and np.all(g.ent_abs == 0)
    # a tie (margin + d+ - d- == 0) is inactive
    cfg49 = stxo.Config(stxo.TRANSE, stxo.L2, 3, 1, 2, margin=49.0)
    assert np.all(stxo.backward(cfg49, stxo.Tables(X), _one(0, 0, 1, [0], [2])).ent == 0)


def test_hinge_pairs_and_k_negatives():
    wl, tabs, bt = small_problem("transe", "l1", b=6, k=3, seed=3)
    cfg = oracle_config(wl)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt)
    pos, neg = fw.scores[:6], fw.scores[6:].reshape(6, 3)
    arg = 1.0 + pos[:, None] - neg                                               # negative (i,kk) pairs with positive i
    np.testing.assert_allclose(fw.hinge_arg.reshape(6, 3), arg, rtol=0, atol=1e-12)
    assert fw.loss == pytest.approx(np.maximum(arg, 0).sum(), rel=1e-14)


# ----------------------------------------------------------------------------- model reductions
def test_transh_reductions():
    wl, tabs, bt = small_problem("transh", "l2", seed=4)
    cfg = oracle_config(wl)
    # both algebraic forms of Sec. 4.5: h_perp + d_r - t_perp == (h-t) + d_r - (w.(h-t)) w
    E, D, Wn = (tabs[k].astype(np.float64) for k in ("ent", "rel", "w"))
    hh = np.concatenate([bt.h, bt.nh]); tt = np.concatenate([bt.t, bt.nt]); rr = np.concatenate([bt.r, np.repeat(bt.r, bt.k)])
    hp = E[hh] - np.sum(Wn[rr] * E[hh], 1, keepdims=True) * Wn[rr]
    tp = E[tt] - np.sum(Wn[rr] * E[tt], 1, keepdims=True) * Wn[rr]
    want = np.linalg.norm(hp + D[rr] - tp, axis=1)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt)
    np.testing.assert_allclose(fw.scores, want, rtol=1e-6)                       # x = h-t is rounded to fp32 first
    # w = 0: a pure translation by d_r, i.e. TransE with relation embedding d_r
    z = dict(tabs, w=np.zeros_like(tabs["w"]))
    fw0 = stxo.forward(cfg, oracle_tables(z), bt)
    cfg_e = stxo.Config(stxo.TRANSE, stxo.L2, wl.n_ent, wl.n_rel, wl.dim)
    fwe = stxo.forward(cfg_e, stxo.Tables(np.concatenate([tabs["ent"], tabs["rel"]])), bt)
    np.testing.assert_allclose(fw0.scores, fwe.scores, rtol=1e-6)
    # w orthogonal to h-t: the projection term vanishes
    E2 = np.zeros((4, 4), np.float32); E2[0] = [1, 2, 0, 0]; E2[1] = [0.5, -1, 0, 0]
    w2 = np.array([[0, 0, 1, 0]], np.float32); d2 = np.array([[0.25, 0.5, 2, 0]], np.float32)
    cfg2 = stxo.Config(stxo.TRANSH, stxo.L1, 4, 1, 4)
    s = stxo.forward(cfg2, stxo.Tables(E2, d2, w2), _one(0, 0, 1)).scores[0]
    assert s == 0.75 + 3.5 + 2.0                                                 # |(0.5,3,0,0)+(0.25,0.5,2,0)|_1
    # w along h-t removes that component entirely
    w3 = np.array([[1, 0, 0, 0]], np.float32)
    s3 = stxo.forward(cfg2, stxo.Tables(E2, np.zeros((1, 4), np.float32), w3), _one(0, 0, 1)).scores[0]
    assert s3 == 3.0


def test_transr_identity_projection_is_transe():
    wl, tabs, bt = small_problem("transr", "l2", seed=5)
    eye = np.tile(np.eye(wl.dim, dtype=np.float32), (wl.n_rel, 1, 1))
    cfg = oracle_config(wl, bf16=False)
    fw = stxo.forward(cfg, oracle_tables(dict(tabs, proj=eye)), bt)
    cfg_e = stxo.Config(stxo.TRANSE, stxo.L2, wl.n_ent, wl.n_rel, wl.dim)
    fwe = stxo.forward(cfg_e, stxo.Tables(np.concatenate([tabs["ent"], tabs["rel"]])), bt)
    np.testing.assert_allclose(fw.scores, fwe.scores, rtol=1e-6)                 # (h-t)+r vs (h+r)-t in fp32
    g = stxo.backward(cfg, oracle_tables(dict(tabs, proj=eye)), bt)
    ge = stxo.backward(cfg_e, stxo.Tables(np.concatenate([tabs["ent"], tabs["rel"]])), bt)
    np.testing.assert_allclose(g.ent, ge.ent[:wl.n_ent], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(g.rel, ge.ent[wl.n_ent:], rtol=1e-5, atol=1e-6)


def test_transr_rectangular_projection_against_numpy():
    wl, tabs, bt = small_problem("transr", "l1", dim=8, rel_dim=5, seed=6)
    cfg = oracle_config(wl, bf16=False)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt)
    hh = np.concatenate([bt.h, bt.nh]); tt = np.concatenate([bt.t, bt.nt]); rr = np.concatenate([bt.r, np.repeat(bt.r, bt.k)])
    E, R, M = (tabs[k].astype(np.float64) for k in ("ent", "rel", "proj"))
    # Eq. 2, unrearranged: M h + r - M t
    y = np.einsum("nkd,nd->nk", M[rr], E[hh]) + R[rr] - np.einsum("nkd,nd->nk", M[rr], E[tt])
    np.testing.assert_allclose(fw.scores, np.abs(y).sum(1), rtol=1e-6)


# ----------------------------------------------------------------------------- gradients
def _loss_of(cfg, tabs, bt):
    return stxo.forward(cfg, oracle_tables(tabs), bt, want_x=False).loss


CASES = [("transe", "l1"), ("transe", "l2"), ("toruse", "torus_l1"), ("toruse", "torus_l2"),
         ("transh", "l2"), ("transh", "l1"), ("transr", "l2"), ("transr", "l1"),
         ("transe", "l2_sq"), ("transh", "l2_sq"), ("transr", "l2_sq")]


@pytest.mark.parametrize("model,dist", CASES)
@pytest.mark.parametrize("reduce", [stxo.SUM, stxo.MEAN])
def test_gradients_by_central_differences(model, dist, reduce):
    # grid=10: table entries are multiples of 2^-10, so x and the perturbed x are exact in fp32
    wl, tabs, bt = small_problem(model, dist, n_ent=10, n_rel=3, b=8, k=2, dim=4,
                                 rel_dim=3 if model == "transr" else None, seed=11, grid=10)
    cfg = oracle_config(wl, reduce=reduce, bf16=False)
    g = stxo.backward(cfg, oracle_tables(tabs), bt)
    eps = 2.0 ** -9
    smooth = dist in ("l2", "torus_l2", "l2_sq") or model in ("transh", "transr")
    for name, grad in (("ent", g.ent), ("rel", g.rel), ("w", g.w), ("proj", g.proj)):
        if grad is None:
            continue
        flat = tabs[name].reshape(-1)
        for idx in range(flat.size):
            keep = flat[idx]
            flat[idx] = keep + np.float32(eps); lp = _loss_of(cfg, tabs, bt)
            flat[idx] = keep - np.float32(eps); lm = _loss_of(cfg, tabs, bt)
            flat[idx] = keep
            fd = (lp - lm) / (2 * eps)
            tol = (2e-3 if smooth else 1e-9) * max(1.0, abs(fd))
            assert abs(fd - grad.reshape(-1)[idx]) <= tol, (name, idx, fd, grad.reshape(-1)[idx])


def _torch_loss(model, dist, reduce, margin, tabs, bt, n_ent, rel_weight=None):
    """The gather formulation with library ops only (index_select + autograd), float64."""
    T = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in tabs.items() if k != "rel_weight"}
    hh = torch.tensor(np.concatenate([bt.h, bt.nh]), dtype=torch.long)
    tt = torch.tensor(np.concatenate([bt.t, bt.nt]), dtype=torch.long)
    rr = torch.tensor(np.concatenate([bt.r, np.repeat(bt.r, bt.k)]), dtype=torch.long)
    E = T["ent"]
    if model in ("transe", "toruse"):
        y = E.index_select(0, hh) + E.index_select(0, n_ent + rr) - E.index_select(0, tt)
    elif model == "transh":
        w, d = T["w"].index_select(0, rr), T["rel"].index_select(0, rr)
        h, t = E.index_select(0, hh), E.index_select(0, tt)
        y = (h - (w * h).sum(1, keepdim=True) * w) + d - (t - (w * t).sum(1, keepdim=True) * w)
    else:
        M = T["proj"].index_select(0, rr)
        y = torch.bmm(M, E.index_select(0, hh).unsqueeze(2)).squeeze(2) + T["rel"].index_select(0, rr) \
            - torch.bmm(M, E.index_select(0, tt).unsqueeze(2)).squeeze(2)
    if dist == "l1":
        s = y.abs().sum(1)
    elif dist == "l2":
        s = (y * y).sum(1).sqrt()
    elif dist == "l2_sq":
        s = (y * y).sum(1)
    else:
        f = y - torch.floor(y)
        m = torch.minimum(f, 1 - f)
        s = m.sum(1) if dist == "torus_l1" else (m * m).sum(1).sqrt()
    if rel_weight is not None:
        s = s * torch.tensor(rel_weight, dtype=torch.float64).index_select(0, rr)
    b, k = bt.b, bt.k
    arg = margin + s[:b].unsqueeze(1) - s[b:].reshape(b, k)
    loss = torch.clamp(arg, min=0).sum()
    if reduce == stxo.MEAN:
        loss = loss / (b * k)
    loss.backward()
    return loss.item(), {k: v.grad.numpy() for k, v in T.items()}


@pytest.mark.parametrize("model,dist", CASES)
@pytest.mark.parametrize("reduce", [stxo.SUM, stxo.MEAN])
def test_gradients_against_library_autograd(model, dist, reduce):
    wl, tabs, bt = small_problem(model, dist, n_ent=40, n_rel=5, b=64, k=2, dim=16,
                                 rel_dim=12 if model == "transr" else None, seed=21, grid=12)
    cfg = oracle_config(wl, reduce=reduce, bf16=False)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt)
    g = stxo.backward(cfg, oracle_tables(tabs), bt)
    loss, tg = _torch_loss(model, dist, reduce, wl.margin, tabs, bt, wl.n_ent)
    assert fw.loss == pytest.approx(loss, rel=1e-12)
    for name, mine in (("ent", g.ent), ("rel", g.rel), ("w", g.w), ("proj", g.proj)):
        if mine is not None:
            np.testing.assert_allclose(mine, tg[name], rtol=1e-9, atol=1e-11, err_msg=name)


@pytest.mark.parametrize("model,dist", [("transe", "l1"), ("transe", "l2"), ("transe", "l2_sq"), ("toruse", "torus_l2"),
                                        ("transh", "l2")])
def test_relation_weight_against_library_autograd(model, dist):
    wl, tabs, bt = small_problem(model, dist, n_ent=40, n_rel=5, b=64, k=2, dim=16, seed=23, grid=12)
    wts = np.array([0.5, 2.0, 1.0, 1.75, 0.25], np.float32)
    cfg = oracle_config(wl, bf16=False)
    tb = oracle_tables(tabs)
    plain_fw = stxo.forward(cfg, tb, bt)
    tb.rel_weight = wts
    fw = stxo.forward(cfg, tb, bt)
    g = stxo.backward(cfg, tb, bt)
    loss, tg = _torch_loss(model, dist, stxo.SUM, wl.margin, tabs, bt, wl.n_ent, rel_weight=wts)
    assert fw.loss == pytest.approx(loss, rel=1e-12) and fw.loss != plain_fw.loss
    rr = np.concatenate([bt.r, np.repeat(bt.r, bt.k)])
    np.testing.assert_allclose(fw.scores, plain_fw.scores * wts[rr].astype(np.float64), rtol=1e-15)
    for name, mine in (("ent", g.ent), ("rel", g.rel), ("w", g.w)):
        if mine is not None:
            np.testing.assert_allclose(mine, tg[name], rtol=1e-9, atol=1e-11, err_msg=name)
    # weights of one change nothing, bit for bit
    tb.rel_weight = np.ones(5, np.float32)
    g1, g0 = stxo.backward(cfg, tb, bt), stxo.backward(cfg, oracle_tables(tabs), bt)
    assert np.array_equal(g1.ent, g0.ent)
    # the column-wise gradient used for spot checks at large sizes sees the weights too
    if cfg.stacked:
        tb.rel_weight = wts
        active = (fw.hinge_arg > 0).astype(np.uint8)
        for col in (0, 7, wl.n_ent + 1):
            want, _ = stxo.grad_column_stacked(cfg, tb, bt, active, col)
            np.testing.assert_allclose(want, g.ent[col], rtol=1e-12, atol=1e-14)


def test_transe_gradient_is_transposed_spmm():
    # Appendix G: dL/dX = A^T dL/dC with C = A X
    wl, tabs, bt = small_problem("transe", "l2", n_ent=20, n_rel=3, b=30, k=2, dim=8, seed=8)
    cfg = oracle_config(wl)
    g = stxo.backward(cfg, oracle_tables(tabs), bt, want_gy=True)
    inc = stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
    at_g = stxo.spmm_csr_t(inc.rowptr, inc.colidx, inc.vals, g.gy.astype(np.float32), wl.n_ent + wl.n_rel)
    np.testing.assert_allclose(g.ent, at_g, rtol=0, atol=1e-5)
    # error scale: sum of |terms| dominates |sum|
    assert np.all(g.ent_abs + 1e-12 >= np.abs(g.ent))


def test_active_override_changes_only_flagged_pairs():
    wl, tabs, bt = small_problem("transe", "l1", b=6, k=1, seed=9)
    cfg = oracle_config(wl)
    none = stxo.backward(cfg, oracle_tables(tabs), bt, active=np.zeros(6, np.uint8))
    assert np.all(none.ent == 0)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt)
    same = stxo.backward(cfg, oracle_tables(tabs), bt, active=(fw.hinge_arg > 0))
    assert np.array_equal(same.ent, stxo.backward(cfg, oracle_tables(tabs), bt).ent)


def test_grad_column_matches_dense_backward():
    wl, tabs, bt = small_problem("toruse", "torus_l1", n_ent=15, n_rel=3, b=40, k=3, dim=8, seed=10)
    cfg = oracle_config(wl)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt)
    g = stxo.backward(cfg, oracle_tables(tabs), bt)
    for col in range(wl.n_ent + wl.n_rel):
        out, aout = stxo.grad_column_stacked(cfg, oracle_tables(tabs), bt, fw.hinge_arg > 0, col)
        np.testing.assert_allclose(out, g.ent[col], rtol=0, atol=1e-12)
        np.testing.assert_allclose(aout, g.ent_abs[col], rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- SGD, wrap, bf16
def test_sgd_closed_form_and_wrap():
    tab = np.array([[1.0, 2.0], [3.0, 4.0]], np.float32)
    stxo.sgd(tab, np.array([[10.0, -20.0], [1.0, 1.0]]), np.array([1, 0], np.uint8), 0.5, 0)
    assert np.array_equal(tab, [[-4.0, 12.0], [3.0, 4.0]])                       # untouched row unchanged
    v = np.array([[-1e-9, 1.25, -0.25, 0.5]], np.float32)
    stxo.sgd(v, np.zeros((1, 4)), np.array([1], np.uint8), 0.1, 1)
    assert np.array_equal(v, [[0.0, 0.25, 0.75, 0.5]])                           # -1e-9 wraps to 1.0f -> 0
    w = np.array([[0.125, 0.0, 2.5]], np.float32); stxo.wrap(w); assert np.array_equal(w, [[0.125, 0.0, 0.5]])
    n = np.array([[3.0, 4.0], [0.0, 0.0]], np.float32)
    stxo.sgd(n, np.zeros((2, 2)), np.array([1, 1], np.uint8), 0.1, 2)
    np.testing.assert_allclose(n, [[0.6, 0.8], [0, 0]], rtol=1e-7)
    # the step is rounded as fp32(lr*g) then subtracted: one triplet, closed form
    x = np.array([[0.1]], np.float32)
    stxo.sgd(x, np.array([[3.0]]), np.array([1], np.uint8), 0.01, 0)
    assert x[0, 0] == np.float32(0.1) - np.float32(np.float32(0.01) * np.float32(3.0))


def test_one_triplet_training_step_closed_form():
    # TransE, L1, one positive (e0 + r -> e1) and one negative (tail e2); all coordinates distinct
    X = np.array([[0.5, -0.25], [0.125, 0.75], [4.0, 4.0], [0.25, 0.25]], np.float32)
    cfg = stxo.Config(stxo.TRANSE, stxo.L1, 3, 1, 2)
    tb = stxo.Tables(X.copy())
    bt = _one(0, 0, 1, [0], [2])
    fw, g = stxo.train_step(cfg, tb, bt, lr=0.5)
    # x+ = (0.625,-0.75) d+=1.375 ; x- = (-3.25,-4) d-=7.25 ; 1+1.375-7.25 < 0 -> inactive
    assert fw.loss == 0.0 and np.array_equal(tb.ent, X)
    cfg2 = stxo.Config(stxo.TRANSE, stxo.L1, 3, 1, 2, margin=10.0)
    fw2, g2 = stxo.train_step(cfg2, tb, bt, lr=0.5)
    assert fw2.loss == 10 + 1.375 - 7.25
    # active: dL/dx+ = sign(x+) = (1,-1); dL/dx- = -sign(x-) = (1,1)
    want = np.zeros((4, 2)); want[0] += [1, -1]; want[3] += [1, -1]; want[1] -= [1, -1]
    want[0] += [1, 1]; want[3] += [1, 1]; want[2] -= [1, 1]
    assert np.array_equal(g2.ent, want)
    assert np.array_equal(tb.ent, X - np.float32(0.5) * want.astype(np.float32))


def test_bf16_rounding_matches_library():
    vals = np.array([1.0, 1 + 2.0**-8, 1 + 2.0**-8 + 2.0**-16, 1 + 3 * 2.0**-8, -0.3, 1e-3, 123456.789, 0.0],
                    np.float32)
    want = torch.tensor(vals).bfloat16().float().numpy()
    got = np.array([stxo.bf16_round(float(v)) for v in vals], np.float32)
    assert np.array_equal(got, want)
    assert got[1] == 1.0 and got[3] == np.float32(1 + 2.0**-6)                   # ties go to even


def test_transr_bf16_mode_rounds_operands_only():
    wl, tabs, bt = small_problem("transr", "l2", seed=12)
    cfg_b = oracle_config(wl, bf16=True)
    cfg_x = oracle_config(wl, bf16=False)
    # tables already representable in bfloat16 -> x = h-t may still need rounding; use tiny integers
    t2 = {k: np.round(v * 4).astype(np.float32) / 4 for k, v in tabs.items()}
    a = stxo.forward(cfg_b, oracle_tables(t2), bt)
    b = stxo.forward(cfg_x, oracle_tables(t2), bt)
    np.testing.assert_array_equal(a.scores, b.scores)
    c = stxo.forward(cfg_b, oracle_tables(tabs), bt)
    d = stxo.forward(cfg_x, oracle_tables(tabs), bt)
    assert not np.array_equal(c.scores, d.scores)
    np.testing.assert_allclose(c.scores, d.scores, rtol=2e-2)
