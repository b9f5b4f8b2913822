"""stx_spmm_semiring_t_static (the entry point that allocates nothing and takes no work buffer: its per-row
terms live in a fixed array inside the library) against stx_spmm_semiring_t, through the C ABI: same bits,
on two calls in a row, the second with a smaller batch, and a refusal beyond the fixed size."""
import numpy as np
import pytest
import torch

from oracle import stxo
from paper_2502_16949_amd import binding as B
from paper_2502_16949_amd import workloads as W
from tests import gpu_util as G
from tests.util import oracle_batch

pytestmark = pytest.mark.gpu


def _problem(n_ent, n_rel, b, k, dim, seed, max_batch):
    wl = W.Workload("case", 7, "transe", "l2", n_ent, n_rel, b, dim, dim, max_batch, k, 1.0, 0.01, 1, 1.1, 1.1)
    h, r, t = W.make_graph(wl.scaled(index=seed))
    tabs = W.make_tables(wl.scaled(index=seed))
    return wl, tabs, oracle_batch(wl, h, r, t, 0, b, seed=seed)


def _both(m, kind, gz):
    rows, dim = m.inc.n_rows, m.cfg.dim
    work = torch.empty(3 * rows * dim, dtype=torch.float32, device=G.DEV)
    m.grads.rows.fill_(float("nan"))
    B.stx_spmm_semiring_t(m.ctx, m.inc, m.params, kind, gz, work, m.grads)
    cols, want = m.grad_rows_numpy()
    m.grads.rows.fill_(float("nan"))
    B.stx_spmm_semiring_t_static(m.ctx, m.inc, m.params, kind, gz, m.grads)
    _, got = m.grad_rows_numpy()
    return cols, want, got


@pytest.mark.parametrize("kind,okind", [(B.STX_COMPLEX, stxo.COMPLEX), (B.STX_DISTMULT, stxo.DISTMULT),
                                        (B.STX_ROTATE, stxo.ROTATE)])
def test_static_scratch_matches_work_buffer_twice(kind, okind):
    dim = 128
    wl, tabs, big = _problem(3000, 40, 5000, 1, dim, seed=41, max_batch=5000)
    _, _, small = _problem(3000, 40, 333, 1, dim, seed=42, max_batch=5000)
    m = G.GpuModel(wl, tabs, max_batch=5000)
    for bt, seed in ((big, 1), (small, 2)):                 # the second call leaves most of the array stale
        m.build(bt)
        gz = np.random.default_rng(seed).uniform(-1, 1, (bt.rows, dim)).astype(np.float32)
        cols, want, got = _both(m, kind, G.dev_f32(gz))
        assert not np.isnan(got).any()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        inc = stxo.build_incidence(bt, wl.n_ent, wl.n_rel)
        ref, scale = stxo.spmm_semiring_t(inc.colidx, tabs["ent"], okind, gz)
        G.check_grad_rows(cols, got, ref, scale, dim, what=f"static semiring {kind}")


def test_static_scratch_refuses_what_does_not_fit():
    # 3 * rows * dim * 4 bytes: 8,192 rows of 1024 floats fill the 96 MiB array exactly
    dim, b = 1024, 4097
    assert 3 * (2 * b) * dim * 4 > B.STX_STATIC_WORK_BYTES == 3 * (2 * 4096) * dim * 4
    wl, tabs, bt = _problem(500, 9, b, 1, dim, seed=43, max_batch=b)
    m = G.GpuModel(wl, tabs, max_batch=b)
    m.build(bt)
    gz = torch.zeros(bt.rows * dim, dtype=torch.float32, device=G.DEV)
    with pytest.raises(B.StxError) as e:
        B.stx_spmm_semiring_t_static(m.ctx, m.inc, m.params, B.STX_COMPLEX, gz, m.grads)
    assert e.value.status == B.STX_ERR_STATIC_LIMIT
    # one positive fewer fits exactly, and runs
    _, _, bt2 = _problem(500, 9, 4096, 1, dim, seed=43, max_batch=b)
    m.build(bt2)
    gz2 = G.dev_f32(np.random.default_rng(5).uniform(-1, 1, bt2.rows * dim))
    cols, want, got = _both(m, B.STX_COMPLEX, gz2)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
