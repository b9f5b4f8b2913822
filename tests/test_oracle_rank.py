"""Pins of the oracle's link-prediction counts (oracle/stxo.c: stxo_rank) that need no GPU: hand-computed
cases, brute force through a library distance routine on exactly representable tables, agreement of the true
entity's score with the training forward pass, and the meaning of the ambiguity band."""
import numpy as np
import pytest
from scipy.spatial.distance import cdist

from oracle import stxo
from tests.util import oracle_config, oracle_tables, small_problem


def _cfg(dist, n_ent, n_rel, dim, model=stxo.TRANSE):
    return stxo.Config(model, dist, n_ent, n_rel, dim)


def test_rank_hand_computed():
    # four entities in the plane, one relation r = (1, 0) stored after them (row n_ent + 0)
    X = np.array([[0, 0], [1, 0], [3, 0], [0, 5], [1, 0]], np.float32)
    h, r = np.array([0, 0, 3], np.int32), np.zeros(3, np.int32)
    t = np.array([1, 2, 2], np.int32)
    # tail side, L1: q = h + r.  (0,r,1): q = (1,0), scores 1,0,2,6 -> true 0, nothing below
    #                            (0,r,2): true 2; entities 1 (0) and 0 (1) are closer
    #                            (3,r,2): q = (1,5), scores 6,5,7,1 -> true 7, all three others closer
    ts, less, band = stxo.rank(_cfg(stxo.L1, 4, 1, 2), X, h, r, t, stxo.TAIL)
    assert ts.tolist() == [0, 2, 7] and less.tolist() == [0, 2, 3] and band.tolist() == [1, 1, 1]
    # head side, L1: q = t - r.  (0,r,1): q = (0,0), scores 0,1,3,5 -> true entity 0 scores 0
    #                            (0,r,2): q = (2,0), scores 2,1,1,7 -> true 2, two closer
    #                            (3,r,2): q = (2,0) -> true entity 3 scores 7, three closer
    ts, less, band = stxo.rank(_cfg(stxo.L1, 4, 1, 2), X, h, r, t, stxo.HEAD)
    assert ts.tolist() == [0, 2, 7] and less.tolist() == [0, 2, 3] and band.tolist() == [1, 1, 1]
    # L2 and its square order the candidates alike; (3,r,2), tail: (1,5)-(3,0) -> sqrt(29)
    ts, less, _ = stxo.rank(_cfg(stxo.L2, 4, 1, 2), X, h, r, t, stxo.TAIL)
    assert ts[2] == pytest.approx(np.sqrt(29.0), rel=1e-15) and less.tolist() == [0, 2, 3]
    ts, less, _ = stxo.rank(_cfg(stxo.L2_SQ, 4, 1, 2), X, h, r, t, stxo.TAIL)
    assert ts.tolist() == [0, 4, 29] and less.tolist() == [0, 2, 3]


def test_rank_exact_ties_are_counted_in_the_band():
    # entities 1 and 2 coincide; entity 3 is as far from q on the other side
    X = np.array([[0, 0], [2, 0], [2, 0], [0, 0], [1, 0]], np.float32)   # last row: r = (1, 0); q = h + r = (1, 0)
    ts, less, band = stxo.rank(_cfg(stxo.L1, 4, 1, 2), X, [0], [0], [1], stxo.TAIL)
    assert ts[0] == 1 and less[0] == 0 and band[0] == 4                  # all four entities are at distance 1
    with pytest.raises(ValueError):
        stxo.rank(stxo.Config(stxo.TRANSR, stxo.L1, 4, 1, 2, 2, bf16_proj=True), stxo.Tables(X[:4], X[4:], None, X[:4].reshape(1, 2, 4)[:, :, :2].copy()),
                  [0], [0], [1], stxo.TAIL)
    with pytest.raises(ValueError):
        stxo.rank(_cfg(stxo.L1, 4, 1, 2), X, [0], [0], [1], 2)


@pytest.mark.parametrize("dist,metric", [(stxo.L1, "cityblock"), (stxo.L2, "sqeuclidean"), (stxo.L2_SQ, "sqeuclidean")])
@pytest.mark.parametrize("side", [stxo.TAIL, stxo.HEAD])
def test_rank_against_library_distance_matrix(dist, metric, side):
    # entries are multiples of 1/2 in [-3, 3): sums, differences and squares are exact in both precisions,
    # so the counts must agree exactly, ties included (a coarse grid makes many)
    rng = np.random.default_rng(11 + dist + side)
    n_ent, n_rel, dim, nq = 200, 5, 4, 80
    X = (rng.integers(-6, 6, (n_ent + n_rel, dim)) / 2.0).astype(np.float32)
    h, t = rng.integers(0, n_ent, nq).astype(np.int32), rng.integers(0, n_ent, nq).astype(np.int32)
    r = rng.integers(0, n_rel, nq).astype(np.int32)
    E, R = X[:n_ent].astype(np.float64), X[n_ent:].astype(np.float64)
    Q = E[h] + R[r] if side == stxo.TAIL else E[t] - R[r]
    D = cdist(Q, E, metric)
    true = D[np.arange(nq), t if side == stxo.TAIL else h]
    ts, less, band = stxo.rank(_cfg(dist, n_ent, n_rel, dim), X, h, r, t, side)
    assert np.array_equal(less, (D < true[:, None]).sum(1))
    assert np.array_equal(band, (D == true[:, None]).sum(1))
    assert band.max() > 1                                                # the case does contain ties
    np.testing.assert_allclose(ts, np.sqrt(true) if dist == stxo.L2 else true, rtol=1e-15)


@pytest.mark.parametrize("dist", [stxo.TORUS_L1, stxo.TORUS_L2])
def test_rank_on_the_torus_brute_force(dist):
    # multiples of 1/64 in [0, 1): fractional parts and their sums are exact
    rng = np.random.default_rng(21 + dist)
    n_ent, n_rel, dim, nq = 150, 4, 5, 60
    X = (rng.integers(0, 64, (n_ent + n_rel, dim)) / 64.0).astype(np.float32)
    h, t = rng.integers(0, n_ent, nq).astype(np.int32), rng.integers(0, n_ent, nq).astype(np.int32)
    r = rng.integers(0, n_rel, nq).astype(np.int32)
    E, R = X[:n_ent].astype(np.float64), X[n_ent:].astype(np.float64)
    for side in (stxo.TAIL, stxo.HEAD):
        Q = E[h] + R[r] if side == stxo.TAIL else E[t] - R[r]
        Y = Q[:, None, :] - E[None, :, :]
        F = Y - np.floor(Y)                                              # the torus distance is even in y
        Mn = np.minimum(F, 1.0 - F)
        D = Mn.sum(2) if dist == stxo.TORUS_L1 else (Mn * Mn).sum(2)
        true = D[np.arange(nq), t if side == stxo.TAIL else h]
        ts, less, band = stxo.rank(_cfg(dist, n_ent, n_rel, dim, stxo.TORUSE), X, h, r, t, side)
        assert np.array_equal(less, (D < true[:, None]).sum(1))
        assert np.array_equal(band, (D == true[:, None]).sum(1))


def test_rank_true_score_is_the_training_score():
    # tail side: the same x = (h + r) - t and the same distance as the forward pass, bit for bit;
    # head side: e - (t - r) differs from it by roundings only
    for model, dist in (("transe", "l1"), ("transe", "l2"), ("toruse", "torus_l1"), ("toruse", "torus_l2")):
        wl, tabs, bt = small_problem(model, dist, n_ent=40, n_rel=5, b=25, k=0, dim=16, seed=3)
        cfg = oracle_config(wl)
        fw = stxo.forward(cfg, oracle_tables(tabs), bt, want_x=False)
        ts, less, band = stxo.rank(cfg, tabs["ent"], bt.h, bt.r, bt.t, stxo.TAIL)
        assert np.array_equal(ts, fw.scores[:25])
        ts_h, _, _ = stxo.rank(cfg, tabs["ent"], bt.h, bt.r, bt.t, stxo.HEAD)
        np.testing.assert_allclose(ts_h, fw.scores[:25], rtol=2e-6)
        assert np.all(band >= 1) and np.all(less + band <= 40)


def test_rank_band_holds_what_single_precision_cannot_order():
    # one dimension, five entities and the relation r = 1 in the last row.  Query (h = 0, r, t = 0): q = 1,
    # the true entity (0) is at distance 1, the others at 1 + 2^-19, 1 - 2^-19, 0.5 and 3
    X = np.array([[0.0], [2.0 + 2.0**-19], [2.0 - 2.0**-19], [1.5], [4.0], [1.0]], np.float32)
    ts, less, band = stxo.rank(_cfg(stxo.L1, 5, 1, 1), X, [0], [0], [0], stxo.TAIL, tol=0.0)
    assert ts[0] == 1.0 and less[0] == 2 and band[0] == 1               # 0.5 and 1 - 2^-19 are closer
    ts, less, band = stxo.rank(_cfg(stxo.L1, 5, 1, 1), X, [0], [0], [0], stxo.TAIL, tol=1e-5)
    assert less[0] == 1 and band[0] == 3                                 # only 0.5 is surely closer
    # the band is symmetric in the two scores and scales with them
    ts, less, band = stxo.rank(_cfg(stxo.L1, 5, 1, 1), X, [0], [0], [0], stxo.TAIL, tol=0.6)
    assert less[0] == 0 and band[0] == 5                                 # |3 - 1| <= 0.6 * 4, |0.5 - 1| <= 0.6 * 1.5


# ------------------------------------------------------------------------------------------ TransH
def _transh_grid_problem(seed, n_ent=120, n_rel=5, dim=4, nq=60):
    """Tables on a coarse grid (multiples of 1/2, normals of small integers): every product and sum of the
    TransH score is exact in single and double precision alike."""
    rng = np.random.default_rng(seed)
    E = (rng.integers(-4, 4, (n_ent, dim)) / 2.0).astype(np.float32)
    D = (rng.integers(-4, 4, (n_rel, dim)) / 2.0).astype(np.float32)
    Wn = rng.integers(-1, 2, (n_rel, dim)).astype(np.float32)
    h, t = rng.integers(0, n_ent, nq).astype(np.int32), rng.integers(0, n_ent, nq).astype(np.int32)
    r = rng.integers(0, n_rel, nq).astype(np.int32)
    return E, D, Wn, h, r, t


@pytest.mark.parametrize("dist", [stxo.L1, stxo.L2_SQ])
@pytest.mark.parametrize("side", [stxo.TAIL, stxo.HEAD])
def test_rank_transh_against_the_projected_form(dist, side):
    # Sec. 4.5 first writes the score with both entities projected onto the relation's hyperplane,
    # h_p + d_r - t_p with v_p = v - (w.v) w; the oracle uses the rearranged form on h - t.  Evaluate the
    # projected form with library array arithmetic for every candidate and count.
    E, D, Wn, h, r, t = _transh_grid_problem(31 + dist + side)
    n_ent, dim = E.shape
    cfg = stxo.Config(stxo.TRANSH, dist, n_ent, D.shape[0], dim)
    ts, less, band = stxo.rank(cfg, stxo.Tables(E, D, Wn), h, r, t, side)
    E64, D64, W64 = E.astype(np.float64), D.astype(np.float64), Wn.astype(np.float64)
    for i in range(len(h)):
        w, dr = W64[r[i]], D64[r[i]]
        proj = lambda v: v - (v @ w)[..., None] * w
        if side == stxo.TAIL:
            Y = proj(E64[h[i]][None, :]) + dr - proj(E64)               # candidates as tails
            true = t[i]
        else:
            Y = proj(E64) + dr - proj(E64[t[i]][None, :])               # candidates as heads
            true = h[i]
        sc = np.abs(Y).sum(1) if dist == stxo.L1 else (Y * Y).sum(1)
        assert ts[i] == sc[true]
        assert less[i] == (sc < sc[true]).sum() and band[i] == (sc == sc[true]).sum()
    assert band.max() > 1


def test_rank_transh_true_score_is_the_training_score_and_zero_normals_give_a_translation():
    wl, tabs, bt = small_problem("transh", "l2", n_ent=40, n_rel=5, b=25, k=0, dim=16, seed=4)
    cfg = oracle_config(wl)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt, want_x=False)
    for side in (stxo.TAIL, stxo.HEAD):
        ts, less, band = stxo.rank(cfg, oracle_tables(tabs), bt.h, bt.r, bt.t, side)
        assert np.array_equal(ts, fw.scores[:25])                        # the same triplet, the same functions
        assert np.all(band >= 1) and np.all(less + band <= 40)
    # w_r = 0: TransH is a translation by d_r, i.e. TransE on the stacked table [E; D] (exact on a grid)
    E, D, Wn, h, r, t = _transh_grid_problem(9)
    n_ent, dim = E.shape
    cfg_h = stxo.Config(stxo.TRANSH, stxo.L1, n_ent, D.shape[0], dim)
    cfg_e = stxo.Config(stxo.TRANSE, stxo.L1, n_ent, D.shape[0], dim)
    for side in (stxo.TAIL, stxo.HEAD):
        got = stxo.rank(cfg_h, stxo.Tables(E, D, np.zeros_like(Wn)), h, r, t, side)
        want = stxo.rank(cfg_e, np.concatenate([E, D]), h, r, t, side)
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
    with pytest.raises(ValueError):
        stxo.rank(stxo.Config(stxo.TRANSR, stxo.L1, n_ent, D.shape[0], dim, dim), stxo.Tables(E, D), h, r, t, 0)   # no M_r


def test_rank_transh_band_uses_the_magnitudes_behind_y():
    # one dimension, w = 1 (so y = d_r whatever the entities are: every candidate ties exactly); with
    # entities of size ~1000 and d_r = 1 a single-precision evaluation cannot order them, and the band,
    # scaled by |x| + |d| + |s w| rather than by the score, says so
    E = np.array([[1000.0], [999.0], [-1000.0]], np.float32)
    D = np.array([[1.0]], np.float32)
    Wn = np.array([[1.0]], np.float32)
    cfg = stxo.Config(stxo.TRANSH, stxo.L1, 3, 1, 1)
    ts, less, band = stxo.rank(cfg, stxo.Tables(E, D, Wn), [0], [0], [1], stxo.TAIL, tol=0.0)
    assert ts[0] == 1.0 and less[0] == 0 and band[0] == 3
    Wn2 = np.array([[1.0 - 2.0**-12]], np.float32)                      # now y = d + x (1 - w^2), x = h - e
    ts, less, band = stxo.rank(cfg, stxo.Tables(E, D, Wn2), [0], [0], [1], stxo.TAIL, tol=0.0)
    assert less[0] == 1 and band[0] == 1                                # e = 0 (x = 0) scores exactly 1, below x = 1
    ts, less, band = stxo.rank(cfg, stxo.Tables(E, D, Wn2), [0], [0], [1], stxo.TAIL, tol=1e-3)
    assert less[0] == 0 and band[0] >= 2                                # scale ~ 2 |x| + 1: 1e-3 of it covers the gap
    # an absolute allowance per query widens the band the same way
    ts, less, band = stxo.rank(cfg, stxo.Tables(E, D, Wn2), [0], [0], [1], stxo.TAIL, tol=0.0, abs_tol=[0.5])
    assert less[0] == 0 and band[0] >= 2


# ------------------------------------------------------------------------------------------ TransR
def _transr_grid_problem(seed, n_ent=90, n_rel=4, dim=4, rel_dim=3, nq=50):
    rng = np.random.default_rng(seed)
    E = (rng.integers(-4, 4, (n_ent, dim)) / 2.0).astype(np.float32)
    Rv = (rng.integers(-4, 4, (n_rel, rel_dim)) / 2.0).astype(np.float32)
    M = rng.integers(-2, 3, (n_rel, rel_dim, dim)).astype(np.float32)
    h, t = rng.integers(0, n_ent, nq).astype(np.int32), rng.integers(0, n_ent, nq).astype(np.int32)
    r = rng.integers(0, n_rel, nq).astype(np.int32)
    return E, Rv, M, h, r, t


@pytest.mark.parametrize("dist", [stxo.L1, stxo.L2_SQ])
@pytest.mark.parametrize("side", [stxo.TAIL, stxo.HEAD])
def test_rank_transr_against_projected_entities(dist, side):
    # Sec. 4.4 scores M_r h + r - M_r t; the oracle applies M_r to h - t.  Project every entity with the
    # library's matrix product, form the score from the projected rows, and count (exact on this grid).
    E, Rv, M, h, r, t = _transr_grid_problem(41 + dist + side)
    n_ent, dim = E.shape
    cfg = stxo.Config(stxo.TRANSR, dist, n_ent, Rv.shape[0], dim, M.shape[1])
    ts, less, band = stxo.rank(cfg, stxo.Tables(E, Rv, None, M), h, r, t, side)
    for i in range(len(h)):
        P = E.astype(np.float64) @ M[r[i]].astype(np.float64).T          # n_ent x rel_dim
        rv = Rv[r[i]].astype(np.float64)
        Y = (P[h[i]] + rv) - P if side == stxo.TAIL else P + rv - P[t[i]]
        true = t[i] if side == stxo.TAIL else h[i]
        sc = np.abs(Y).sum(1) if dist == stxo.L1 else (Y * Y).sum(1)
        assert ts[i] == sc[true]
        assert less[i] == (sc < sc[true]).sum() and band[i] == (sc == sc[true]).sum()
    assert band.max() > 1


def test_rank_transr_true_score_is_the_training_score_and_identity_matrices_give_transe():
    wl, tabs, bt = small_problem("transr", "l2", n_ent=40, n_rel=5, b=25, k=0, dim=8, rel_dim=6, seed=5)
    cfg = oracle_config(wl, bf16=False)
    fw = stxo.forward(cfg, oracle_tables(tabs), bt, want_x=False)
    for side in (stxo.TAIL, stxo.HEAD):
        ts, less, band = stxo.rank(cfg, oracle_tables(tabs), bt.h, bt.r, bt.t, side)
        assert np.array_equal(ts, fw.scores[:25])
    # M_r = I: TransR is TransE on the stacked table [E; R] (Sec. 4.4 with the identity; exact on a grid)
    E, Rv, M, h, r, t = _transr_grid_problem(12, dim=4, rel_dim=4)
    M[:] = np.eye(4, dtype=np.float32)
    n_ent = E.shape[0]
    cfg_r = stxo.Config(stxo.TRANSR, stxo.L1, n_ent, Rv.shape[0], 4, 4)
    cfg_e = stxo.Config(stxo.TRANSE, stxo.L1, n_ent, Rv.shape[0], 4)
    for side in (stxo.TAIL, stxo.HEAD):
        got = stxo.rank(cfg_r, stxo.Tables(E, Rv, None, M), h, r, t, side)
        want = stxo.rank(cfg_e, np.concatenate([E, Rv]), h, r, t, side)
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
