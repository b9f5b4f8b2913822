"""GPU parity for the semiring products of Appendix D (DistMult, ComplEx, RotatE) and their backward:
HIP library through the C ABI against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import stxo
from paper_2502_16949_amd import binding as B
from paper_2502_16949_amd import workloads as W
from tests import gpu_util as G
from tests.util import oracle_batch

pytestmark = pytest.mark.gpu

KINDS = [(B.STX_DISTMULT, stxo.DISTMULT), (B.STX_COMPLEX, stxo.COMPLEX), (B.STX_ROTATE, stxo.ROTATE)]


def _problem(n_ent, n_rel, b, k, dim, seed, zipf=0.0):
    wl = W.Workload("case", 7, "transe", "l2", n_ent, n_rel, b, dim, dim, b, k, 1.0, 0.01, 1, zipf, zipf)
    h, r, t = W.make_graph(wl.scaled(index=seed))
    tabs = W.make_tables(wl.scaled(index=seed))
    bt = oracle_batch(wl, h, r, t, 0, b, seed=seed)
    return wl, tabs, bt


CASES = [
    # n_ent, n_rel, b, k, dim, zipf
    (10, 2, 1, 0, 8, 0.0),            # one row
    (300, 7, 683, 2, 32, 1.1),        # ragged tail, skewed columns, 8 lanes per row
    (1000, 20, 1024, 1, 128, 0.0),    # 32 lanes per row
    (5, 1, 3000, 1, 64, 0.0),         # six columns: every segment spans many tiles of the transposed product
    (2000, 11, 777, 1, 200, 1.1),     # width not a power of two
    (500, 9, 500, 1, 1024, 1.1),      # widest rows: four float4 per lane
]


@pytest.mark.parametrize("n_ent,n_rel,b,k,dim,zipf", CASES)
@pytest.mark.parametrize("kind,okind", KINDS)
def test_semiring_product_bit_exact(kind, okind, n_ent, n_rel, b, k, dim, zipf):
    wl, tabs, bt = _problem(n_ent, n_rel, b, k, dim, seed=b + dim, zipf=zipf)
    m = G.GpuModel(wl, tabs)
    m.build(bt)
    z = torch.full((m.inc.n_rows, dim), float("nan"), dtype=torch.float32, device=G.DEV)
    B.stx_spmm_semiring(m.ctx, m.inc, m.params, kind, z)
    torch.cuda.synchronize()
    inc = stxo.build_incidence(bt, n_ent, n_rel)
    want = stxo.spmm_semiring(inc.colidx, tabs["ent"], okind)
    got = z.cpu().numpy()
    assert np.array_equal(got, want)                       # every product and sum rounded once, same order


@pytest.mark.parametrize("n_ent,n_rel,b,k,dim,zipf", CASES)
@pytest.mark.parametrize("kind,okind", KINDS)
def test_semiring_backward(kind, okind, n_ent, n_rel, b, k, dim, zipf):
    wl, tabs, bt = _problem(n_ent, n_rel, b, k, dim, seed=b + dim + 1, zipf=zipf)
    m = G.GpuModel(wl, tabs)
    m.build(bt)
    rows = m.inc.n_rows
    gz = np.random.default_rng(b).uniform(-1, 1, (rows, dim)).astype(np.float32)
    work = torch.empty(3 * rows * dim, dtype=torch.float32, device=G.DEV)
    m.grads.rows.fill_(float("nan"))
    B.stx_spmm_semiring_t(m.ctx, m.inc, m.params, kind, G.dev_f32(gz), work, m.grads)
    cols, got = m.grad_rows_numpy()
    inc = stxo.build_incidence(bt, n_ent, n_rel)
    ref, scale = stxo.spmm_semiring_t(inc.colidx, tabs["ent"], okind, gz)
    assert np.array_equal(cols, inc.touched_cols)
    G.check_grad_rows(cols, got, ref, scale, dim, what=f"semiring {kind}")
    # bitwise reproducible: fixed summation order, no atomics
    B.stx_spmm_semiring_t(m.ctx, m.inc, m.params, kind, G.dev_f32(gz), work, m.grads)
    _, again = m.grad_rows_numpy()
    assert np.array_equal(got.view(np.uint32), again.view(np.uint32))


def test_semiring_repeated_columns_in_a_row_and_empty_batch():
    wl, tabs, bt = _problem(40, 3, 64, 1, 16, seed=3)
    bt = stxo.Batch(bt.h, bt.r, bt.h, bt.nh, bt.nh)        # head == tail in every row
    m = G.GpuModel(wl, tabs)
    m.build(bt)
    rows, dim = m.inc.n_rows, 16
    inc = stxo.build_incidence(bt, 40, 3)
    gz = np.random.default_rng(1).uniform(-1, 1, (rows, dim)).astype(np.float32)
    work = torch.empty(3 * rows * dim, dtype=torch.float32, device=G.DEV)
    for kind, okind in KINDS:
        z = torch.empty(rows, dim, dtype=torch.float32, device=G.DEV)
        B.stx_spmm_semiring(m.ctx, m.inc, m.params, kind, z)
        assert np.array_equal(z.cpu().numpy(), stxo.spmm_semiring(inc.colidx, tabs["ent"], okind))
        B.stx_spmm_semiring_t(m.ctx, m.inc, m.params, kind, G.dev_f32(gz), work, m.grads)
        cols, got = m.grad_rows_numpy()
        ref, scale = stxo.spmm_semiring_t(inc.colidx, tabs["ent"], okind, gz)
        G.check_grad_rows(cols, got, ref, scale, dim, what=f"semiring {kind}")
    e = np.empty(0, np.int32)
    m.build(stxo.Batch(e, e, e, e, e))
    z = torch.zeros(4, dtype=torch.float32, device=G.DEV)
    B.stx_spmm_semiring(m.ctx, m.inc, m.params, B.STX_COMPLEX, z)
    B.stx_spmm_semiring_t(m.ctx, m.inc, m.params, B.STX_COMPLEX, z, work, m.grads)
    torch.cuda.synchronize()


def test_semiring_rejects_bad_arguments():
    wl, tabs, bt = _problem(40, 3, 8, 1, 16, seed=4)
    m = G.GpuModel(wl, tabs)
    m.build(bt)
    z = torch.empty(m.inc.n_rows * 16, dtype=torch.float32, device=G.DEV)
    with pytest.raises(B.StxError) as e:
        B.stx_spmm_semiring(m.ctx, m.inc, m.params, 3, z)
    assert e.value.status == B.STX_ERR_BAD_ARG
    wlh = W.Workload("case", 7, "transh", "l2", 40, 3, 8, 16, 16, 8, 1, 1.0, 0.01, 1, 0.0, 0.0)
    mh = G.GpuModel(wlh, W.make_tables(wlh))
    mh.build(bt)
    with pytest.raises(B.StxError) as e:
        B.stx_spmm_semiring(mh.ctx, mh.inc, mh.params, B.STX_DISTMULT, z)
    assert e.value.status == B.STX_ERR_UNSUPPORTED
