"""ctypes front end of the CPU oracle (oracle/stxo.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the cpu_baseline
leg of bench.py.  Nothing in the product package imports it, and it imports nothing from the
product package.  Argument marshalling only; all arithmetic is in stxo.c.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stxo.c")
_LIB = os.path.join(_HERE, "libstxo.so")

TRANSE, TRANSH, TRANSR, TORUSE = 0, 1, 2, 3
L1, L2, TORUS_L1, TORUS_L2, L2_SQ = 0, 1, 2, 3, 4
SUM, MEAN = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-ffp-contract=off", "-fno-fast-math", "-shared",
             "-fPIC", _SRC, "-o", _LIB, "-lm"])
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("model", C.c_int32), ("dist", C.c_int32), ("reduce", C.c_int32),
                ("dim", C.c_int32), ("rel_dim", C.c_int32),
                ("n_ent", C.c_int64), ("n_rel", C.c_int64),
                ("margin", C.c_float), ("bf16_proj", C.c_int32)]


class _Tables(C.Structure):
    _fields_ = [("ent", C.c_void_p), ("rel", C.c_void_p), ("w", C.c_void_p), ("proj", C.c_void_p),
                ("rel_weight", C.c_void_p)]


class _Batch(C.Structure):
    _fields_ = [("h", C.c_void_p), ("r", C.c_void_p), ("t", C.c_void_p),
                ("nh", C.c_void_p), ("nt", C.c_void_p), ("b", C.c_int32), ("k", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.stxo_rng_u64.restype = C.c_uint64
        _lib.stxo_rng_u64.argtypes = [C.c_uint64, C.c_uint64]
        _lib.stxo_bf16_round.restype = C.c_float
        _lib.stxo_bf16_round.argtypes = [C.c_float]
        _lib.stxo_sample_negatives.restype = None
        _lib.stxo_sample_negatives.argtypes = [C.c_void_p] * 3 + [C.c_int64, C.c_int32, C.c_int64,
                                                                  C.c_uint64, C.c_uint64, C.c_int64,
                                                                  C.c_int64, C.c_void_p, C.c_void_p]
        _lib.stxo_build_incidence.restype = C.c_int
        _lib.stxo_build_incidence.argtypes = [C.c_void_p, C.c_int64, C.c_int64] + [C.c_void_p] * 9
        _lib.stxo_spmm_csr.restype = None
        _lib.stxo_spmm_csr.argtypes = [C.c_int64] + [C.c_void_p] * 4 + [C.c_int32, C.c_void_p]
        _lib.stxo_spmm_semiring.restype = C.c_int
        _lib.stxo_spmm_semiring.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        _lib.stxo_spmm_semiring_t.restype = C.c_int
        _lib.stxo_spmm_semiring_t.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 3
        _lib.stxo_rank.restype = C.c_int
        _lib.stxo_rank.argtypes = [C.c_void_p] * 5 + [C.c_int64, C.c_int32, C.c_double] + [C.c_void_p] * 4
        _lib.stxo_spmm_csr_t.restype = None
        _lib.stxo_spmm_csr_t.argtypes = [C.c_int64] + [C.c_void_p] * 4 + [C.c_int32, C.c_void_p]
        _lib.stxo_forward.restype = C.c_int
        _lib.stxo_forward.argtypes = [C.c_void_p] * 7
        _lib.stxo_backward.restype = C.c_int
        _lib.stxo_backward.argtypes = [C.c_void_p] * 14
        _lib.stxo_sgd.restype = None
        _lib.stxo_sgd.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                  C.c_float, C.c_int32]
        _lib.stxo_wrap.restype = None
        _lib.stxo_wrap.argtypes = [C.c_void_p, C.c_int64]
        _lib.stxo_grad_column_stacked.restype = C.c_int
        _lib.stxo_grad_column_stacked.argtypes = [C.c_void_p] * 4 + [C.c_int64, C.c_void_p, C.c_void_p]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


@dataclass
class Config:
    model: int
    dist: int
    n_ent: int
    n_rel: int
    dim: int
    rel_dim: int = 0
    margin: float = 1.0
    reduce: int = SUM
    bf16_proj: bool = False

    def c(self) -> _Cfg:
        return _Cfg(self.model, self.dist, self.reduce, self.dim, self.rel_dim or self.dim,
                    self.n_ent, self.n_rel, self.margin, int(self.bf16_proj))

    @property
    def stacked(self) -> bool:
        return self.model in (TRANSE, TORUSE)

    @property
    def out_dim(self) -> int:
        return (self.rel_dim or self.dim) if self.model == TRANSR else self.dim


class Batch:
    """b positives and b*k negatives, host int32 arrays."""

    def __init__(self, h, r, t, nh, nt):
        self.h, self.r, self.t, self.nh, self.nt = map(_i32, (h, r, t, nh, nt))
        self.b = int(self.h.shape[0])
        self.k = int(self.nh.shape[0] // self.b) if self.b else 0
        assert self.nh.shape[0] == self.b * self.k == self.nt.shape[0]

    @property
    def rows(self) -> int:
        return self.b * (1 + self.k)

    def c(self) -> _Batch:
        return _Batch(_p(self.h), _p(self.r), _p(self.t), _p(self.nh), _p(self.nt), self.b, self.k)


class Tables:
    def __init__(self, ent, rel=None, w=None, proj=None, rel_weight=None):
        self.ent, self.rel, self.w, self.proj = _f32(ent), _f32(rel), _f32(w), _f32(proj)
        self.rel_weight = _f32(rel_weight)      # fixed per-relation weight of the distance (TransM), or None

    def c(self) -> _Tables:
        return _Tables(_p(self.ent), _p(self.rel), _p(self.w), _p(self.proj), _p(self.rel_weight))

    def copy(self) -> "Tables":
        cp = lambda a: None if a is None else a.copy()
        return Tables(cp(self.ent), cp(self.rel), cp(self.w), cp(self.proj), cp(self.rel_weight))


def rng_u64(seed: int, counter: int) -> int:
    return int(lib().stxo_rng_u64(seed & (2**64 - 1), counter & (2**64 - 1)))


def bf16_round(v: float) -> float:
    return float(lib().stxo_bf16_round(v))


def sample_negatives(h, r, t, k, n_ent, seed, epoch=0, m_total=None, global_offset=0):
    h, r, t = _i32(h), _i32(r), _i32(t)
    m = h.shape[0]
    m_total = m if m_total is None else m_total
    nh = np.empty(m * k, np.int32)
    nt = np.empty(m * k, np.int32)
    lib().stxo_sample_negatives(_p(h), _p(r), _p(t), m, k, n_ent, seed, epoch, m_total, global_offset,
                                _p(nh), _p(nt))
    return nh, nt


@dataclass
class Incidence:
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray
    touched_cols: np.ndarray
    seg_ptr: np.ndarray
    row_idx: np.ndarray
    sign: np.ndarray
    seg_id: np.ndarray
    n_touched: int


def build_incidence(bt: Batch, n_ent: int, n_rel: int) -> Incidence:
    rows, nnz = bt.rows, 3 * bt.rows
    cap = min(nnz, n_ent + n_rel)
    rowptr = np.empty(rows + 1, np.int32)
    colidx = np.empty(nnz, np.int32)
    vals = np.empty(nnz, np.float32)
    touched = np.empty(cap, np.int32)
    seg_ptr = np.empty(cap + 1, np.int32)
    row_idx = np.empty(nnz, np.int32)
    sign = np.empty(nnz, np.int8)
    seg_id = np.empty(nnz, np.int32)
    n_touched = C.c_int32(0)
    cb = bt.c()
    rc = lib().stxo_build_incidence(C.byref(cb), n_ent, n_rel, _p(rowptr), _p(colidx), _p(vals),
                                    _p(touched), _p(seg_ptr), _p(row_idx), _p(sign), _p(seg_id),
                                    C.byref(n_touched))
    if rc != 0:
        raise ValueError(f"stxo_build_incidence failed with code {rc}")
    u = n_touched.value
    return Incidence(rowptr, colidx, vals, touched[:u].copy(), seg_ptr[:u + 1].copy(), row_idx, sign,
                     seg_id, u)


def spmm_csr(rowptr, colidx, vals, X, nrows=None):
    X = _f32(X)
    nrows = len(rowptr) - 1 if nrows is None else nrows
    d = X.shape[1]
    out = np.empty((nrows, d), np.float32)
    lib().stxo_spmm_csr(nrows, _p(_i32(rowptr)), _p(_i32(colidx)), _p(_f32(vals)), _p(X), d, _p(out))
    return out


DISTMULT, COMPLEX, ROTATE = 0, 1, 2


def spmm_semiring(colidx, X, kind: int):
    """The semiring products of the paper's Appendix D over rows of three columns (head, relation, tail)."""
    X = _f32(X)
    colidx = _i32(colidx)
    nrows, d = colidx.shape[0] // 3, X.shape[1]
    out = np.empty((nrows, d), np.float32)
    if lib().stxo_spmm_semiring(nrows, _p(colidx), _p(X), d, kind, _p(out)) != 0:
        raise ValueError("stxo_spmm_semiring: bad kind or odd width for a complex kind")
    return out


def spmm_semiring_t(colidx, X, kind: int, G):
    """Gradient of a real loss with respect to X through the semiring product, given G = dL/dZ: (gradient,
    error scale), both (rows of X) x d in float64."""
    X, G = _f32(X), _f32(G)
    colidx = _i32(colidx)
    out = np.zeros(X.shape, np.float64)
    scale = np.zeros(X.shape, np.float64)
    if lib().stxo_spmm_semiring_t(colidx.shape[0] // 3, _p(colidx), _p(X), X.shape[1], kind, _p(G), _p(out),
                                  _p(scale)) != 0:
        raise ValueError("stxo_spmm_semiring_t: bad kind or odd width for a complex kind")
    return out, scale


TAIL, HEAD = 0, 1


def rank(cfg: "Config", tables, h, r, t, side: int, tol: float = 0.0, abs_tol=None):
    """Raw link-prediction counts of every test triplet against all entities: (true_score float64,
    n_less int64, n_band int64); see stxo_rank in stxo.c.  tables: a Tables object, or the stacked table
    X = [E;R] of TransE / TorusE as an array."""
    if not isinstance(tables, Tables):
        tables = Tables(_f32(tables))
    if cfg.model == TRANSH and (tables.rel is None or tables.w is None):
        raise ValueError("stxo_rank: TransH needs the d_r and w_r tables")
    if cfg.model == TRANSR and (tables.rel is None or tables.proj is None):
        raise ValueError("stxo_rank: TransR needs the r and M_r tables")
    h, r, t = _i32(h), _i32(r), _i32(t)
    nq = h.shape[0]
    ts = np.empty(nq, np.float64)
    less = np.empty(nq, np.int64)
    band = np.empty(nq, np.int64)
    cc, ct = cfg.c(), tables.c()
    if abs_tol is not None:
        abs_tol = np.ascontiguousarray(abs_tol, dtype=np.float64)
        assert abs_tol.shape == (nq,)
    if lib().stxo_rank(C.byref(cc), C.byref(ct), _p(h), _p(r), _p(t), nq, side, tol, _p(abs_tol), _p(ts), _p(less),
                       _p(band)) != 0:
        raise ValueError("stxo_rank: side 0 (tail) or 1 (head); TransR without bfloat16 operand rounding")
    return ts, less, band


def spmm_csr_t(rowptr, colidx, vals, G, ncols):
    G = _f32(G)
    nrows, d = G.shape
    out = np.zeros((ncols, d), np.float64)
    lib().stxo_spmm_csr_t(nrows, _p(_i32(rowptr)), _p(_i32(colidx)), _p(_f32(vals)), _p(G), d, _p(out))
    return out


@dataclass
class Forward:
    x: np.ndarray          # rows x dim, fp32: (h+r)-t or h-t
    scores: np.ndarray     # rows, float64
    hinge_arg: np.ndarray  # b*k, float64: margin + d_pos - d_neg
    loss: float


def forward(cfg: Config, tb: Tables, bt: Batch, want_x: bool = True) -> Forward:
    x = np.empty((bt.rows, cfg.dim), np.float32) if want_x else None
    scores = np.empty(bt.rows, np.float64)
    arg = np.empty(bt.b * bt.k, np.float64)
    loss = C.c_double(0)
    cc, ct, cb = cfg.c(), tb.c(), bt.c()
    rc = lib().stxo_forward(C.byref(cc), C.byref(ct), C.byref(cb), _p(x), _p(scores), _p(arg),
                            C.byref(loss))
    if rc != 0:
        raise RuntimeError(f"stxo_forward failed with code {rc}")
    return Forward(x, scores, arg, loss.value)


@dataclass
class Grads:
    ent: np.ndarray
    ent_abs: np.ndarray
    rel: np.ndarray | None = None
    rel_abs: np.ndarray | None = None
    w: np.ndarray | None = None
    w_abs: np.ndarray | None = None
    proj: np.ndarray | None = None
    proj_abs: np.ndarray | None = None
    gy: np.ndarray | None = None
    ambiguous: np.ndarray | None = None   # per row: an L1-kind subgradient of TransH/TransR sits on a jump


def backward(cfg: Config, tb: Tables, bt: Batch, active=None, want_gy: bool = False) -> Grads:
    d, kd = cfg.dim, cfg.rel_dim or cfg.dim
    z = lambda *s: np.zeros(s, np.float64)
    n_rows_ent = cfg.n_ent + (cfg.n_rel if cfg.stacked else 0)
    g = Grads(z(n_rows_ent, d), z(n_rows_ent, d))
    if cfg.model == TRANSH:
        g.rel, g.rel_abs, g.w, g.w_abs = z(cfg.n_rel, d), z(cfg.n_rel, d), z(cfg.n_rel, d), z(cfg.n_rel, d)
    elif cfg.model == TRANSR:
        g.rel, g.rel_abs = z(cfg.n_rel, kd), z(cfg.n_rel, kd)
        g.proj, g.proj_abs = z(cfg.n_rel, kd, d), z(cfg.n_rel, kd, d)
    if want_gy:
        g.gy = np.empty((bt.rows, cfg.out_dim), np.float64)
    act = None if active is None else np.ascontiguousarray(active, dtype=np.uint8)
    g.ambiguous = np.zeros(bt.rows, np.uint8)
    cc, ct, cb = cfg.c(), tb.c(), bt.c()
    rc = lib().stxo_backward(C.byref(cc), C.byref(ct), C.byref(cb), _p(act),
                             _p(g.ent), _p(g.ent_abs), _p(g.rel), _p(g.rel_abs), _p(g.w), _p(g.w_abs),
                             _p(g.proj), _p(g.proj_abs), _p(g.gy), _p(g.ambiguous))
    if rc != 0:
        raise RuntimeError(f"stxo_backward failed with code {rc}")
    return g


def sgd(table: np.ndarray, grad: np.ndarray, touched: np.ndarray, lr: float, mode: int = 0) -> None:
    """In place on `table` (fp32, C-contiguous).  mode 0 plain, 1 torus wrap, 2 renormalise rows."""
    assert table.dtype == np.float32 and table.flags.c_contiguous
    t2 = table.reshape(touched.shape[0], -1)
    grad = np.ascontiguousarray(grad, dtype=np.float64).reshape(t2.shape)
    touched = np.ascontiguousarray(touched, dtype=np.uint8)
    lib().stxo_sgd(_p(table), t2.shape[0], t2.shape[1], _p(grad), _p(touched), lr, mode)


def wrap(table: np.ndarray) -> None:
    assert table.dtype == np.float32 and table.flags.c_contiguous
    lib().stxo_wrap(_p(table), table.size)


def grad_column_stacked(cfg: Config, tb: Tables, bt: Batch, active, col: int):
    out = np.empty(cfg.dim, np.float64)
    aout = np.empty(cfg.dim, np.float64)
    act = np.ascontiguousarray(active, dtype=np.uint8)
    cc, ct, cb = cfg.c(), tb.c(), bt.c()
    rc = lib().stxo_grad_column_stacked(C.byref(cc), C.byref(ct), C.byref(cb), _p(act), col, _p(out),
                                        _p(aout))
    if rc != 0:
        raise RuntimeError(f"stxo_grad_column_stacked failed with code {rc}")
    return out, aout


def touched_masks(cfg: Config, bt: Batch):
    """Which table rows a batch touches: (entity-table mask, relation mask)."""
    ent = np.zeros(cfg.n_ent + (cfg.n_rel if cfg.stacked else 0), np.uint8)
    rel = np.zeros(cfg.n_rel, np.uint8)
    for a in (bt.h, bt.t, bt.nh, bt.nt):
        ent[a] = 1
    rel[bt.r] = 1
    if cfg.stacked:
        ent[cfg.n_ent + bt.r] = 1
    return ent, rel


def train_step(cfg: Config, tb: Tables, bt: Batch, lr: float, renorm_w: bool = True):
    """One full step on the oracle's own tables (updated in place).  Returns (Forward, Grads)."""
    fw = forward(cfg, tb, bt, want_x=False)
    g = backward(cfg, tb, bt)
    m_ent, m_rel = touched_masks(cfg, bt)
    sgd(tb.ent, g.ent, m_ent, lr, 1 if cfg.model == TORUSE else 0)
    if cfg.model == TRANSH:
        sgd(tb.rel, g.rel, m_rel, lr, 0)
        sgd(tb.w, g.w, m_rel, lr, 2 if renorm_w else 0)
    elif cfg.model == TRANSR:
        sgd(tb.rel, g.rel, m_rel, lr, 0)
        sgd(tb.proj, g.proj, m_rel, lr, 0)
    return fw, g
