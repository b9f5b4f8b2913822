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


def check_incidence(got: dict, want: stxo.Incidence, transpose_only=False):
    """Bit-exact comparison of every integer structure of A and A^T (transpose_only: of A^T alone, for a
    step that has already written the next batch's A)."""
    assert got["n_touched"] == want.n_touched
    names = ("rowptr", "colidx", "vals", "touched_cols", "seg_ptr", "row_idx", "sign", "seg_id")
    for name in names[3:] if transpose_only else names:
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


USAGE = []               # (what, largest share of its bar that any tightly checked element used), per check
HEADROOM = 0.5           # a check fails when an element uses more than this share of its bar


def check_grad_rows(cols, rows, g_dense, g_abs, width, tol=REL_TOL, what="rows", all_cols=None, allowance=None,
                    headroom=HEADROOM):
    """Row-sparse GPU gradient against the oracle's dense table: elementwise within tol * sum|terms|,
    and in the infinity norm within tol * ||ref||_inf.  all_cols: every column the GPU listed (when
    `cols` is a subset of them), for the check that unlisted columns received nothing.
    allowance (dense, like g_dense; optional): elements where it is nonzero may be off by that much more
    (see ambiguous_allowance).  All other elements must stay within `headroom` of the bar, so that the bar is
    visibly not what makes the check pass; the largest share used is returned and recorded in USAGE."""
    ref = g_dense[cols][:, :width]
    scale = g_abs[cols][:, :width]
    if len(cols) == 0:
        return 0.0
    extra = np.zeros_like(ref) if allowance is None else allowance[cols][:, :width]
    err = np.abs(rows[:, :width].astype(np.float64) - ref)
    bad = err > tol * scale + extra + 1e-30
    assert not bad.any(), (what, int(bad.sum()), float(err.max()), float((err / (scale + 1e-30)).max()))
    tight = extra == 0
    used = float((err[tight] / (tol * scale[tight] + 1e-30)).max()) if tight.any() else 0.0
    USAGE.append((what, used))
    assert used <= headroom, (what, used)
    if tight.any():
        assert err[tight].max() <= tol * max(np.abs(ref).max(), 1e-30) + 1e-30, (what, err.max(), np.abs(ref).max())
    # columns not in the touched list received nothing
    mask = np.ones(g_dense.shape[0], bool)
    mask[cols if all_cols is None else all_cols] = False
    assert not np.any(g_abs[mask]), what
    return used


def pair_coefficients(active, b, k, mean):
    """|coefficient| of every row's dL/dy from the hinge flags: positives sum their active pairs."""
    scale = 1.0 / (b * k) if mean else 1.0
    act = np.asarray(active, np.float64).reshape(b, k) * scale
    return np.concatenate([act.sum(1), act.reshape(-1)])


def ambiguous_allowance(wl, tabs, bt, active, amb, mean, bf16=False):
    """TransH / TransR with an L1-kind norm: in a row the oracle flags as ambiguous some computed y_j sits within
    rounding of a jump of the subgradient, so the fp32 evaluation may take another branch there and that element
    of dL/dy differs by up to 2 |coef| of the row.  Pushed through the row's backward formulas (Sec. 4.4, 4.5),
    that bounds how far every gradient element fed by such a row may move; the bound is added to the bar of
    exactly those elements.  Returns dense arrays {"ent", "rel", "w" | "proj"} (zeros where no flagged row
    contributes), or None when no row is flagged."""
    idx = np.nonzero(amb)[0]
    if len(idx) == 0:
        return None
    hh = np.concatenate([bt.h, bt.nh])[idx]; tt = np.concatenate([bt.t, bt.nt])[idx]
    rr = np.concatenate([bt.r, np.repeat(bt.r, bt.k)])[idx]
    c2 = 2.0 * pair_coefficients(active, bt.b, bt.k, mean)[idx]
    x = (tabs["ent"][hh] - tabs["ent"][tt]).astype(np.float64)
    out = {"ent": np.zeros((wl.n_ent, wl.dim)), "rel": np.zeros((wl.n_rel, wl.rel_dim if wl.model == "transr" else wl.dim))}
    np.add.at(out["rel"], rr, c2[:, None] * np.ones(out["rel"].shape[1]))
    if wl.model == "transh":
        w = tabs["w"].astype(np.float64)[rr]
        w1 = np.abs(w).sum(1, keepdims=True)
        s = np.abs((w * x).sum(1, keepdims=True))
        gx = c2[:, None] * (1.0 + w1 * np.abs(w))                  # d gx = d gy - (d gy . w) w
        out["w"] = np.zeros((wl.n_rel, wl.dim))
        np.add.at(out["w"], rr, c2[:, None] * (w1 * np.abs(x) + s))   # d gw = -((d gy . w) x + s d gy)
    else:
        rnd = (lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32)).bfloat16().float().numpy()) if bf16 else (lambda a: a)
        M = np.abs(rnd(tabs["proj"]).astype(np.float64))
        xq = np.abs(rnd(x.astype(np.float32)).astype(np.float64))
        gx = c2[:, None] * M[rr].sum(1)                            # d gx = M^T d gy
        out["proj"] = np.zeros((wl.n_rel, wl.rel_dim, wl.dim))
        np.add.at(out["proj"], rr, c2[:, None, None] * np.ones((1, wl.rel_dim, 1)) * xq[:, None, :])   # d gM = d gy x^T
    np.add.at(out["ent"], hh, gx)
    np.add.at(out["ent"], tt, gx)
    return out
