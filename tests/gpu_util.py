"""Drives the HIP library through its C ABI for the GPU parity tests and compares with the oracle."""
from __future__ import annotations

import numpy as np
import torch

from oracle import stxo
from paper_2502_16949_amd import binding as B
from paper_2502_16949_amd import workloads as W

DEV = "cuda:0"
REL_TOL = 1e-5          # fp32 bar for scores, loss, gradients and updated tables


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


class GpuModel:
    """One context + tables + scratch outputs for a workload-like description."""

    def __init__(self, wl: W.Workload, tabs: dict, reduce=B.STX_SUM, flags=0, max_batch=None, max_neg=None):
        self.wl = wl
        self.cfg = B.make_config(wl.model, wl.dist, wl.n_ent, wl.n_rel, wl.dim, max_batch or wl.batch,
                                 wl.n_neg if max_neg is None else max_neg, rel_dim=wl.rel_dim, margin=wl.margin,
                                 reduce=reduce, flags=flags)
        self.ctx = B.Context(self.cfg, DEV)
        self.params = B.Params(*(None if tabs.get(k) is None else dev_f32(tabs[k])
                                 for k in ("ent", "rel", "w", "proj", "rel_weight")))
        self.inc = B.Incidence(self.ctx)
        self.grads = B.Grads(self.ctx)
        self.scores = torch.empty(self.ctx.rows_max, dtype=torch.float32, device=DEV)
        self.loss = torch.zeros(1, dtype=torch.float32, device=DEV)

    def build(self, bt: stxo.Batch):
        self.h, self.r, self.t = dev_i32(bt.h), dev_i32(bt.r), dev_i32(bt.t)
        self.nh, self.nt = dev_i32(bt.nh), dev_i32(bt.nt)
        B.stx_build_incidence(self.ctx, self.h, self.r, self.t, self.nh if bt.k else None,
                              self.nt if bt.k else None, bt.k, self.inc)

    def forward(self):
        B.stx_forward(self.ctx, self.inc, self.params, self.scores, self.loss)

    def backward(self):
        B.stx_backward(self.ctx, self.inc, self.params, self.grads)

    def sgd(self, lr):
        B.stx_sgd_step(self.ctx, self.params, self.inc, self.grads, lr)

    def backward_sgd(self, lr, with_grads=True):
        B.stx_backward_sgd(self.ctx, self.inc, self.params, self.grads if with_grads else None, lr)

    # -- results as numpy -------------------------------------------------------------------------
    def incidence_numpy(self):
        torch.cuda.synchronize()
        inc, rows, nnz = self.inc, self.inc.n_rows, self.inc.nnz
        u = int(inc.n_touched.item())
        g = lambda t, n: t[:n].cpu().numpy()
        return dict(rowptr=g(inc.a_rowptr, rows + 1), colidx=g(inc.a_colidx, nnz), vals=g(inc.a_vals, nnz),
                    touched_cols=g(inc.at_touched_cols, u), seg_ptr=g(inc.at_seg_ptr, u + 1),
                    row_idx=g(inc.at_row_idx, nnz), sign=g(inc.at_sign, nnz), seg_id=g(inc.at_seg_id, nnz),
                    packed=g(inc.at_packed, nnz), n_touched=u)

    def scores_numpy(self):
        torch.cuda.synchronize()
        return self.scores[:self.inc.n_rows].cpu().numpy(), float(self.loss.item())

    def grad_rows_numpy(self):
        torch.cuda.synchronize()
        u = int(self.inc.n_touched.item())
        return self.inc.at_touched_cols[:u].cpu().numpy(), self.grads.rows[:u].cpu().numpy()


def check_incidence(got: dict, want: stxo.Incidence):
    """Bit-exact comparison of every integer structure of A and A^T."""
    assert got["n_touched"] == want.n_touched
    for name in ("rowptr", "colidx", "vals", "touched_cols", "seg_ptr", "row_idx", "sign", "seg_id"):
        w = getattr(want, name)
        assert got[name].dtype == w.dtype, name
        assert np.array_equal(got[name], w), name
    head = np.zeros(len(want.row_idx), np.int32)
    head[want.seg_ptr[:-1]] = 1
    packed = (want.row_idx << 2) | (head << 1) | (want.sign < 0).astype(np.int32)
    assert np.array_equal(got["packed"], packed), "packed"


def gpu_active_flags(scores: np.ndarray, b: int, k: int, margin: float) -> np.ndarray:
    """The hinge decision exactly as the kernel takes it: fp32, (margin + d_pos) - d_neg > 0."""
    s = scores.astype(np.float32)
    pos = np.repeat(s[:b], k) if k else s[:0]
    arg = (np.float32(margin) + pos).astype(np.float32) - s[b:b + b * k]
    return arg > 0


def check_scores_and_loss(scores, loss, fw: stxo.Forward, reduce_mean: bool, tol=REL_TOL):
    np.testing.assert_allclose(scores, fw.scores, rtol=tol, atol=0)
    # the loss is a sum of non-negative hinge terms; near-tie terms contribute <= tol * scale each
    assert abs(loss - fw.loss) <= tol * max(abs(fw.loss), 1e-30) + 1e-30, (loss, fw.loss)


def resolve_active(scores, fw: stxo.Forward, bt: stxo.Batch, margin: float, tol=REL_TOL):
    """GPU hinge flags; they must agree with the oracle's except on near ties
    (|margin + d+ - d-| <= tol * (margin + d+ + d-)), where either outcome is accepted."""
    act_gpu = gpu_active_flags(scores, bt.b, bt.k, margin)
    act_ref = fw.hinge_arg > 0
    dpos = np.repeat(fw.scores[:bt.b], bt.k)
    dneg = fw.scores[bt.b:]
    near = np.abs(fw.hinge_arg) <= tol * (margin + dpos + dneg)
    assert np.array_equal(act_gpu[~near], act_ref[~near])
    return act_gpu


def check_grad_rows(cols, rows, g_dense, g_abs, width, tol=REL_TOL, what="rows", all_cols=None):
    """Row-sparse GPU gradient against the oracle's dense table: elementwise within tol * sum|terms|,
    and in the infinity norm within tol * ||ref||_inf.  all_cols: every column the GPU listed (when
    `cols` is a subset of them), for the check that unlisted columns received nothing."""
    ref = g_dense[cols][:, :width]
    scale = g_abs[cols][:, :width]
    if len(cols) == 0:
        return
    err = np.abs(rows[:, :width].astype(np.float64) - ref)
    bad = err > tol * scale + 1e-30
    assert not bad.any(), (what, int(bad.sum()), float(err.max()), float((err / (scale + 1e-30)).max()))
    assert err.max() <= tol * max(np.abs(ref).max(), 1e-30) + 1e-30, (what, err.max(), np.abs(ref).max())
    # columns not in the touched list received nothing
    mask = np.ones(g_dense.shape[0], bool)
    mask[cols if all_cols is None else all_cols] = False
    assert not np.any(g_abs[mask]), what
