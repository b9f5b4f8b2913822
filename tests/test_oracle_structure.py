"""Pins of the oracle's integer side: random numbers, negative sampler, incidence matrix, and the
generic sparse products (paper Sec. 4.2, Appendices B and G).  No GPU needed."""
import os

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.stats import chisquare

from oracle import stxo
from tests.util import small_problem


def _read(path):
    with open(path) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


# ----------------------------------------------------------------------------- random numbers
def test_splitmix64_known_answers(golden_dir):
    for ln in _read(os.path.join(golden_dir, "splitmix64_kat.txt")):
        seed, idx, val = map(int, ln.split())
        assert stxo.rng_u64(seed, idx) == val


def test_rng_is_counter_based_and_uniform():
    # any output is addressable directly, and differs between neighbouring counters and seeds
    a = [stxo.rng_u64(42, i) for i in range(2000)]
    assert len(set(a)) == 2000
    assert stxo.rng_u64(43, 0) != stxo.rng_u64(42, 0)
    u = np.array(a, dtype=np.uint64)
    # chi-square on the top byte and on the low byte
    for shift in (56, 0):
        cnt = np.bincount(((u >> np.uint64(shift)) & np.uint64(0xFF)).astype(np.int64), minlength=256)
        assert chisquare(cnt).pvalue > 1e-4


# ----------------------------------------------------------------------------- negative sampler
def test_negatives_follow_the_stated_mapping():
    rng = np.random.default_rng(1)
    n_ent, m, k, seed, epoch, m_total, off = 977, 300, 3, 5, 2, 1000, 123
    h = rng.integers(0, n_ent, m).astype(np.int32)
    t = rng.integers(0, n_ent, m).astype(np.int32)
    r = rng.integers(0, 7, m).astype(np.int32)
    nh, nt = stxo.sample_negatives(h, r, t, k, n_ent, seed, epoch, m_total, off)
    for i in range(m):
        for kk in range(k):
            ctr = (epoch * m_total + off + i) * k + kk     # Python integers: no overflow involved
            u = stxo.rng_u64(seed, ctr)
            e = ((u & 0xFFFFFFFF) * n_ent) >> 32
            if u >> 63:
                assert (nh[i * k + kk], nt[i * k + kk]) == (e, t[i])
            else:
                assert (nh[i * k + kk], nt[i * k + kk]) == (h[i], e)


def test_negatives_statistics():
    n_ent, m, k = 50, 40000, 1
    h = np.full(m, 3, np.int32)
    t = np.full(m, 7, np.int32)
    r = np.zeros(m, np.int32)
    nh, nt = stxo.sample_negatives(h, r, t, k, n_ent, seed=9)
    head_side = nt == 7
    tail_side = nh == 3
    assert np.all(head_side | tail_side)                      # exactly one side is replaced
    frac = np.mean(nh != 3)                                   # p = 1/2, minus chance hits of entity 3
    assert abs(frac - 0.5 * (1 - 1 / n_ent)) < 0.01
    repl = np.where(nh != 3, nh, nt)
    assert repl.min() >= 0 and repl.max() < n_ent
    assert chisquare(np.bincount(nh[nh != 3], minlength=n_ent)[np.arange(n_ent) != 3]).pvalue > 1e-4
    # pre-generated once: the same (seed, epoch) gives the same negatives; another epoch differs
    nh2, nt2 = stxo.sample_negatives(h, r, t, k, n_ent, seed=9)
    assert np.array_equal(nh, nh2) and np.array_equal(nt, nt2)
    nh3, _ = stxo.sample_negatives(h, r, t, k, n_ent, seed=9, epoch=1)
    assert not np.array_equal(nh, nh3)


def test_negatives_batches_agree_with_whole():
    rng = np.random.default_rng(3)
    n_ent, m, k = 100, 64, 2
    h, t = (rng.integers(0, n_ent, m).astype(np.int32) for _ in range(2))
    r = np.zeros(m, np.int32)
    nh, nt = stxo.sample_negatives(h, r, t, k, n_ent, seed=1)
    nh_b, nt_b = stxo.sample_negatives(h[16:48], r[16:48], t[16:48], k, n_ent, seed=1, m_total=m,
                                       global_offset=16)
    assert np.array_equal(nh[16 * k:48 * k], nh_b) and np.array_equal(nt[16 * k:48 * k], nt_b)


# ----------------------------------------------------------------------------- incidence matrix
def test_paper_worked_examples(golden_dir):
    for ln in _read(os.path.join(golden_dir, "incidence_examples.txt")):
        left, right = ln.split("|")
        form, n_ent, n_rel, h, r, t = left.split()
        n_ent, n_rel, h, r, t = map(int, (n_ent, n_rel, h, r, t))
        want = {}
        tok = right.split()
        for c, v in zip(tok[::2], tok[1::2]):
            want[int(c)] = float(v)
        # one positive and no negatives
        bt = stxo.Batch([h], [r], [t], np.empty(0, np.int32), np.empty(0, np.int32))
        inc = stxo.build_incidence(bt, n_ent, n_rel)
        cols, vals = inc.colidx[:3], inc.vals[:3]
        if form == "ht":
            cols, vals = cols[[0, 2]], vals[[0, 2]]            # the ht view: slots 0 and 2
        assert dict(zip(cols.tolist(), vals.tolist())) == want


def _dense(inc, rows, ncol):
    a = np.zeros((rows, ncol))
    for i in range(rows):
        for p in range(inc.rowptr[i], inc.rowptr[i + 1]):
            a[i, inc.colidx[p]] += inc.vals[p]
    return a


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_incidence_invariants_and_bruteforce(seed):
    wl, _, bt = small_problem("transe", "l1", n_ent=17, n_rel=3, b=15, k=2, seed=seed)
    if seed == 2:                                             # force self-loops: h == t stays two entries
        bt = stxo.Batch(bt.h, bt.r, bt.h, bt.nh, bt.nt)
    n_ent, n_rel, rows = wl.n_ent, wl.n_rel, bt.rows
    inc = stxo.build_incidence(bt, n_ent, n_rel)
    nnz = 3 * rows
    assert np.array_equal(inc.rowptr, 3 * np.arange(rows + 1))         # exactly three per row
    assert np.array_equal(inc.vals.reshape(rows, 3), np.tile([1, 1, -1], (rows, 1)))
    # row layout: positives first, negative (i,kk) at b + i*k + kk with the positive's relation
    hh = np.concatenate([bt.h, bt.nh]); tt = np.concatenate([bt.t, bt.nt])
    rr = np.concatenate([bt.r, np.repeat(bt.r, bt.k)])
    assert np.array_equal(inc.colidx.reshape(rows, 3), np.stack([hh, n_ent + rr, tt], 1))
    dense = _dense(inc, rows, n_ent + n_rel)
    assert np.all(dense.sum(1) == 1)                                    # +1 +1 -1
    assert np.all(dense[:, :n_ent].sum(1) == 0)                         # ht view sums to zero
    # column sums of A = (#head) + (#relation) - (#tail)
    want = (np.bincount(hh, minlength=n_ent + n_rel) + np.bincount(n_ent + rr, minlength=n_ent + n_rel)
            - np.bincount(tt, minlength=n_ent + n_rel))
    assert np.array_equal(dense.sum(0), want)
    # transpose structure against a stable library sort of the column ids
    order = np.argsort(inc.colidx, kind="stable")
    assert np.array_equal(inc.row_idx, order // 3)
    assert np.array_equal(inc.sign, np.where(order % 3 == 2, -1, 1))
    cols_sorted = inc.colidx[order]
    uniq, first = np.unique(cols_sorted, return_index=True)
    assert inc.n_touched == len(uniq)
    assert np.array_equal(inc.touched_cols, uniq)
    assert np.array_equal(inc.seg_ptr, np.append(first, nnz))
    assert np.array_equal(inc.touched_cols[inc.seg_id], cols_sorted)
    # dense transpose rebuilt from the compressed form equals dense.T
    at = np.zeros((n_ent + n_rel, rows))
    for s in range(inc.n_touched):
        for e in range(inc.seg_ptr[s], inc.seg_ptr[s + 1]):
            at[inc.touched_cols[s], inc.row_idx[e]] += inc.sign[e]
    assert np.array_equal(at, dense.T)


def test_incidence_rejects_bad_indices():
    bt = stxo.Batch([5], [0], [99], np.empty(0, np.int32), np.empty(0, np.int32))
    with pytest.raises(ValueError):
        stxo.build_incidence(bt, 10, 2)


def test_density_is_three_per_row_for_a_complete_graph():
    # every ordered pair of 6 entities, one relation: a fully dense graph still gives 3 nnz per row
    n = 6
    h, t = map(np.ravel, np.meshgrid(np.arange(n), np.arange(n), indexing="ij"))
    bt = stxo.Batch(h, np.zeros(n * n, np.int32), t, np.empty(0, np.int32), np.empty(0, np.int32))
    inc = stxo.build_incidence(bt, n, 1)
    assert np.all(np.diff(inc.rowptr) == 3) and len(inc.colidx) == 3 * n * n


# ----------------------------------------------------------------------------- A.X and A^T.G
def test_spmm_equals_h_plus_r_minus_t_bitwise():
    wl, tabs, bt = small_problem("transe", "l1", n_ent=40, n_rel=5, b=50, k=2, dim=16, seed=4)
    inc = stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
    X = tabs["ent"]
    C = stxo.spmm_csr(inc.rowptr, inc.colidx, inc.vals, X)
    hh = np.concatenate([bt.h, bt.nh]); tt = np.concatenate([bt.t, bt.nt])
    rr = np.concatenate([bt.r, np.repeat(bt.r, bt.k)])
    want = (X[hh] + X[wl.n_ent + rr]) - X[tt]                  # numpy fp32, same order of operations
    assert C.dtype == np.float32 and np.array_equal(C, want)
    # the model forward returns the same x
    cfg = stxo.Config(stxo.TRANSE, stxo.L1, wl.n_ent, wl.n_rel, wl.dim)
    fw = stxo.forward(cfg, stxo.Tables(X), bt)
    assert np.array_equal(fw.x, want)
    # ht view: slots 0 and 2 only
    ht_ptr = 2 * np.arange(bt.rows + 1, dtype=np.int32)
    ht_col = inc.colidx.reshape(-1, 3)[:, [0, 2]].ravel()
    ht_val = inc.vals.reshape(-1, 3)[:, [0, 2]].ravel()
    Cht = stxo.spmm_csr(ht_ptr, ht_col, ht_val, X[:wl.n_ent])
    assert np.array_equal(Cht, X[hh] - X[tt])
    cfg_h = stxo.Config(stxo.TRANSH, stxo.L2, wl.n_ent, wl.n_rel, wl.dim)
    z = np.zeros((wl.n_rel, wl.dim), np.float32)
    fwh = stxo.forward(cfg_h, stxo.Tables(X[:wl.n_ent], z, z), bt)
    assert np.array_equal(fwh.x, X[hh] - X[tt])


def test_spmm_closed_forms_and_library():
    wl, _, bt = small_problem("transe", "l1", n_ent=40, n_rel=5, b=30, k=1, dim=4, seed=5)
    inc = stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
    ncol = wl.n_ent + wl.n_rel
    ones = np.ones((ncol, 4), np.float32)
    assert np.all(stxo.spmm_csr(inc.rowptr, inc.colidx, inc.vals, ones) == 1.0)
    ramp = np.tile(np.arange(ncol, dtype=np.float32)[:, None], (1, 4))
    hh = np.concatenate([bt.h, bt.nh]); tt = np.concatenate([bt.t, bt.nt])
    rr = np.concatenate([bt.r, np.repeat(bt.r, bt.k)])
    got = stxo.spmm_csr(inc.rowptr, inc.colidx, inc.vals, ramp)
    assert np.array_equal(got[:, 0], (hh + wl.n_ent + rr - tt).astype(np.float32))
    X = np.random.default_rng(0).standard_normal((ncol, 4)).astype(np.float32)
    A = sp.csr_matrix((inc.vals.astype(np.float64), inc.colidx, inc.rowptr), shape=(bt.rows, ncol))
    np.testing.assert_allclose(stxo.spmm_csr(inc.rowptr, inc.colidx, inc.vals, X), A @ X.astype(np.float64),
                               rtol=0, atol=1e-6)


def test_transposed_product_adjoint_and_library():
    wl, _, bt = small_problem("transe", "l1", n_ent=25, n_rel=4, b=40, k=2, dim=6, seed=6)
    inc = stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
    ncol = wl.n_ent + wl.n_rel
    rng = np.random.default_rng(1)
    X = rng.standard_normal((ncol, 6)).astype(np.float32)
    G = rng.standard_normal((bt.rows, 6)).astype(np.float32)
    A = sp.csr_matrix((inc.vals.astype(np.float64), inc.colidx, inc.rowptr), shape=(bt.rows, ncol))
    AtG = stxo.spmm_csr_t(inc.rowptr, inc.colidx, inc.vals, G, ncol)
    np.testing.assert_allclose(AtG, A.T @ G.astype(np.float64), rtol=1e-13, atol=1e-13)
    lhs = np.sum((A @ X.astype(np.float64)) * G)              # <A X, G>
    rhs = np.sum(X.astype(np.float64) * AtG)                  # <X, A^T G>
    assert abs(lhs - rhs) <= 1e-10 * abs(lhs)
    # the same product from the compressed transpose (what the GPU kernel walks)
    out = np.zeros((ncol, 6))
    for s in range(inc.n_touched):
        for e in range(inc.seg_ptr[s], inc.seg_ptr[s + 1]):
            out[inc.touched_cols[s]] += float(inc.sign[e]) * G[inc.row_idx[e]].astype(np.float64)
    np.testing.assert_allclose(out, AtG, rtol=1e-13, atol=1e-13)


def test_appendix_two_by_two_expansion():
    # Appendix G: dL/dx1 = a1 dL/dc1 + a3 dL/dc3, dL/dx2 = a1 dL/dc2 + a3 dL/dc4,
    #             dL/dx3 = a2 dL/dc1 + a4 dL/dc3, dL/dx4 = a2 dL/dc2 + a4 dL/dc4
    a1, a2, a3, a4 = 2.0, -3.0, 5.0, 7.0
    dc1, dc2, dc3, dc4 = 0.5, -1.5, 2.25, 4.0
    rowptr = np.array([0, 2, 4], np.int32)
    colidx = np.array([0, 1, 0, 1], np.int32)
    vals = np.array([a1, a2, a3, a4], np.float32)
    G = np.array([[dc1, dc2], [dc3, dc4]], np.float32)
    out = stxo.spmm_csr_t(rowptr, colidx, vals, G, 2)
    want = np.array([[a1 * dc1 + a3 * dc3, a1 * dc2 + a3 * dc4], [a2 * dc1 + a4 * dc3, a2 * dc2 + a4 * dc4]])
    assert np.array_equal(out, want)


# ----------------------------------------------------------------------------- Appendix D semirings
def test_semiring_products_hand_computed():
    # one row (h, r, t) = columns (0, 1, 2) of a table of width 2 = one complex number per row
    X = np.array([[1, 2], [3, 4], [5, -6]], np.float32)                  # h = 1+2i, r = 3+4i, t = 5-6i
    col = np.array([0, 1, 2], np.int32)
    assert np.array_equal(stxo.spmm_semiring(col, X, stxo.DISTMULT)[0], [15, -48])   # 1*3*5, 2*4*(-6)
    # (1+2i)(3+4i) = -5+10i;  times conj(t) = 5+6i:  (-5+10i)(5+6i) = -25-60 + (-30+50)i = -85+20i
    assert np.array_equal(stxo.spmm_semiring(col, X, stxo.COMPLEX)[0], [-85, 20])
    # RotatE: h r - t = -5+10i - (5-6i) = -10+16i
    assert np.array_equal(stxo.spmm_semiring(col, X, stxo.ROTATE)[0], [-10, 16])
    with pytest.raises(ValueError):
        stxo.spmm_semiring(col, np.ones((3, 3), np.float32), stxo.COMPLEX)             # odd width


def test_semiring_products_against_library_complex_arithmetic():
    rng = np.random.default_rng(3)
    n, d, rows = 40, 16, 200
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    col = rng.integers(0, n, 3 * rows).astype(np.int32)
    h, r, t = (X[col[s::3]].astype(np.float64) for s in range(3))
    np.testing.assert_allclose(stxo.spmm_semiring(col, X, stxo.DISTMULT), h * r * t, rtol=3e-7, atol=1e-7)
    cx = lambda a: a[:, 0::2] + 1j * a[:, 1::2]
    for kind, want in ((stxo.COMPLEX, cx(h) * cx(r) * np.conj(cx(t))), (stxo.ROTATE, cx(h) * cx(r) - cx(t))):
        got = stxo.spmm_semiring(col, X, kind).astype(np.float64)
        np.testing.assert_allclose(got[:, 0::2], want.real, rtol=0, atol=1e-6)
        np.testing.assert_allclose(got[:, 1::2], want.imag, rtol=0, atol=1e-6)
    # a unit relation leaves DistMult / ComplEx as h t / h conj(t), and a rotation by r = 1 gives h - t
    X[1] = np.tile([1, 0], d // 2)
    col2 = np.array([0, 1, 2], np.int32)
    np.testing.assert_array_equal(stxo.spmm_semiring(col2, X, stxo.ROTATE)[0], X[0] - X[2])
    z = stxo.spmm_semiring(col2, X, stxo.COMPLEX)[0].astype(np.float64)
    want = cx(X[0:1].astype(np.float64)) * np.conj(cx(X[2:3].astype(np.float64)))
    np.testing.assert_allclose(z[0::2], want.real[0], atol=1e-6)


def test_semiring_backward_hand_computed():
    # one row over columns (0, 1, 2), one complex number per table row, dL/dz = g = 1 + i
    X = np.array([[1, 2], [3, 4], [5, -6]], np.float32)                  # h = 1+2i, r = 3+4i, t = 5-6i
    col = np.array([0, 1, 2], np.int32)
    G = np.array([[1, 1]], np.float32)
    # DistMult, element by element: dh = g r t = (15, -24), dr = g h t = (5, -12), dt = g h r = (3, 8)
    out, scale = stxo.spmm_semiring_t(col, X, stxo.DISTMULT, G)
    assert np.array_equal(out, [[15, -24], [5, -12], [3, 8]])
    assert np.array_equal(scale, np.abs(out))
    # ComplEx: dh = g conj(r) t = (1+i)(3-4i)(5-6i) = (7-i)(5-6i) = 29-47i
    #          dr = g conj(h) t = (1+i)(1-2i)(5-6i) = (3-i)(5-6i) = 9-23i
    #          dt = conj(g) h r = (1-i)(-5+10i) = 5+15i
    out, _ = stxo.spmm_semiring_t(col, X, stxo.COMPLEX, G)
    assert np.array_equal(out, [[29, -47], [9, -23], [5, 15]])
    # RotatE: dh = g conj(r) = (1+i)(3-4i) = 7-i, dr = g conj(h) = (1+i)(1-2i) = 3-i, dt = -g
    out, scale = stxo.spmm_semiring_t(col, X, stxo.ROTATE, G)
    assert np.array_equal(out, [[7, -1], [3, -1], [-1, -1]])
    assert np.array_equal(scale, [[14, 14], [6, 6], [2, 2]])             # (1+1)(3+4), (1+1)(1+2), 1+1


def test_semiring_backward_against_library_autograd():
    # the library differentiates L = sum(G * Z) through its own complex arithmetic; repeated columns inside a
    # row (h = t, h = r) and across rows exercise the accumulation
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    n, d, rows = 12, 8, 60
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    col = rng.integers(0, n, 3 * rows).astype(np.int32)
    col[0:3] = [4, 4, 4]
    col[3:6] = [2, 7, 2]
    G = rng.uniform(-1, 1, (rows, d)).astype(np.float32)
    idx = [torch.from_numpy(col[s::3].astype(np.int64)) for s in range(3)]
    Gt = torch.from_numpy(G.astype(np.float64))
    for kind in (stxo.DISTMULT, stxo.COMPLEX, stxo.ROTATE):
        Xt = torch.from_numpy(X.astype(np.float64)).requires_grad_(True)
        if kind == stxo.DISTMULT:
            z = Xt[idx[0]] * Xt[idx[1]] * Xt[idx[2]]
            loss = (Gt * z).sum()
        else:
            Xc = torch.view_as_complex(Xt.reshape(n, d // 2, 2))
            h, r, t = Xc[idx[0]], Xc[idx[1]], Xc[idx[2]]
            z = h * r * t.conj() if kind == stxo.COMPLEX else h * r - t
            loss = (Gt * torch.view_as_real(z).reshape(rows, d)).sum()
        loss.backward()
        out, scale = stxo.spmm_semiring_t(col, X, kind, G)
        np.testing.assert_allclose(out, Xt.grad.numpy(), rtol=0, atol=1e-12)
        assert np.all(scale >= np.abs(out) - 1e-12)


def test_semiring_backward_is_the_directional_derivative():
    # Z is linear in every table row that a matrix row names once: <G, Z(X + eps D) - Z(X - eps D)> / (2 eps)
    # equals <dL/dX, D> up to the cubic term, with Z from the forward oracle
    rng = np.random.default_rng(6)
    n, d, rows = 30, 8, 50
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    col = rng.integers(0, n, 3 * rows).astype(np.int32)
    G = rng.uniform(-1, 1, (rows, d)).astype(np.float32)
    D = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    eps = np.float32(2.0**-6)                                            # X +- eps D is exact enough in fp32
    for kind in (stxo.DISTMULT, stxo.COMPLEX, stxo.ROTATE):
        zp = stxo.spmm_semiring(col, X + eps * D, kind).astype(np.float64)
        zm = stxo.spmm_semiring(col, X - eps * D, kind).astype(np.float64)
        fd = np.sum(G * (zp - zm)) / (2.0 * float(eps))
        out, _ = stxo.spmm_semiring_t(col, X, kind, G)
        assert abs(fd - np.sum(out * D)) <= 2e-3 * max(1.0, abs(fd))
