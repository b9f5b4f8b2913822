"""Thin ctypes binding of libstx (include/stx.h): same names, argument marshalling only.

PyTorch is used for device memory and the stream; every step of the method runs in the library's
HIP kernels.  There is no CPU fallback: if libstx.so is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstx.so")

STX_OK = 0
STX_ERR_NULL, STX_ERR_BAD_ARG, STX_ERR_INDEX_RANGE, STX_ERR_WORKSPACE = 1, 2, 3, 4
STX_ERR_STATE, STX_ERR_UNSUPPORTED, STX_ERR_HIP, STX_ERR_STATIC_LIMIT = 5, 6, 7, 8
STX_STATIC_WORK_BYTES = 96 << 20
STX_TRANSE, STX_TRANSH, STX_TRANSR, STX_TORUSE = 0, 1, 2, 3
STX_L1, STX_L2, STX_TORUS_L1, STX_TORUS_L2, STX_L2_SQ = 0, 1, 2, 3, 4
STX_SUM, STX_MEAN = 0, 1
STX_FLAG_RENORM_W, STX_FLAG_BF16_PROJ = 1, 2
STX_DISTMULT, STX_COMPLEX, STX_ROTATE = 0, 1, 2
STX_TAIL, STX_HEAD = 0, 1

MODELS = {"transe": STX_TRANSE, "transh": STX_TRANSH, "transr": STX_TRANSR, "toruse": STX_TORUSE}
DISTS = {"l1": STX_L1, "l2": STX_L2, "torus_l1": STX_TORUS_L1, "torus_l2": STX_TORUS_L2, "l2_sq": STX_L2_SQ}

EXPORTS = ["stx_workspace_bytes", "stx_create", "stx_destroy", "stx_sample_negatives", "stx_build_incidence",
           "stx_check_indices", "stx_spmm", "stx_spmm_semiring", "stx_spmm_semiring_t", "stx_spmm_semiring_t_static", "stx_rank", "stx_rank_work_bytes", "stx_forward", "stx_backward", "stx_sgd_step", "stx_backward_sgd", "stx_train_step", "stx_profile_kernel",
           "stx_profile_every", "stx_profile_read", "stx_profile_dump", "stx_copy_f32", "stx_read_sectors", "stx_status_string"]


class StxError(RuntimeError):
    def __init__(self, call: str, status: int):
        self.status = status
        super().__init__(f"{call}: {status_string(status)} (status {status})")


class stx_config(C.Structure):
    _fields_ = [("model", C.c_int32), ("dist", C.c_int32), ("reduce", C.c_int32), ("dim", C.c_int32),
                ("rel_dim", C.c_int32), ("n_ent", C.c_int64), ("n_rel", C.c_int64), ("margin", C.c_float),
                ("max_batch", C.c_int32), ("max_neg", C.c_int32), ("flags", C.c_uint32)]


class stx_params(C.Structure):
    _fields_ = [("ent", C.c_void_p), ("rel", C.c_void_p), ("w", C.c_void_p), ("proj", C.c_void_p),
                ("rel_weight", C.c_void_p)]


class stx_incidence(C.Structure):
    _fields_ = [("b", C.c_int32), ("k", C.c_int32), ("n_rows", C.c_int64), ("nnz", C.c_int64),
                ("a_rowptr", C.c_void_p), ("a_colidx", C.c_void_p), ("a_vals", C.c_void_p),
                ("at_touched_cols", C.c_void_p), ("at_seg_ptr", C.c_void_p), ("at_row_idx", C.c_void_p),
                ("at_sign", C.c_void_p), ("at_seg_id", C.c_void_p), ("at_packed", C.c_void_p),
                ("n_touched", C.c_void_p)]


class stx_grads(C.Structure):
    _fields_ = [("rows", C.c_void_p), ("w_rows", C.c_void_p), ("proj", C.c_void_p)]


class stx_batch(C.Structure):
    _fields_ = [("h", C.c_void_p), ("r", C.c_void_p), ("t", C.c_void_p), ("b", C.c_int32), ("k", C.c_int32),
                ("seed", C.c_uint64), ("epoch", C.c_uint64), ("m_total", C.c_int64), ("global_offset", C.c_int64),
                ("neg_h", C.c_void_p), ("neg_t", C.c_void_p), ("next", C.c_void_p)]


_lib = None


def lib():
    """Load libstx.so from the package directory.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2502_16949_amd.build); "
                               "there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
        L.stx_workspace_bytes.argtypes = [C.POINTER(stx_config), C.POINTER(C.c_size_t)]
        L.stx_create.argtypes = [C.POINTER(stx_config), vp, C.c_size_t, vp, C.POINTER(vp)]
        L.stx_destroy.argtypes = [vp]
        L.stx_sample_negatives.argtypes = [vp, vp, vp, vp, i64, i32, u64, u64, i64, i64, vp, vp]
        L.stx_build_incidence.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, C.POINTER(stx_incidence)]
        L.stx_check_indices.argtypes = [vp, C.POINTER(i64)]
        L.stx_spmm.argtypes = [vp, C.POINTER(stx_incidence), C.POINTER(stx_params), vp]
        L.stx_spmm_semiring.argtypes = [vp, C.POINTER(stx_incidence), C.POINTER(stx_params), i32, vp]
        L.stx_spmm_semiring_t.argtypes = [vp, C.POINTER(stx_incidence), C.POINTER(stx_params), i32, vp, vp,
                                          C.POINTER(stx_grads)]
        L.stx_spmm_semiring_t_static.argtypes = [vp, C.POINTER(stx_incidence), C.POINTER(stx_params), i32, vp,
                                                 C.POINTER(stx_grads)]
        L.stx_rank.argtypes = [vp, C.POINTER(stx_params), vp, vp, vp, i64, i32, vp, vp, vp, vp, C.c_size_t]
        L.stx_rank_work_bytes.argtypes = [vp, i64, C.POINTER(C.c_size_t)]
        L.stx_forward.argtypes = [vp, C.POINTER(stx_incidence), C.POINTER(stx_params), vp, vp]
        L.stx_backward.argtypes = [vp, C.POINTER(stx_incidence), C.POINTER(stx_params), C.POINTER(stx_grads)]
        L.stx_sgd_step.argtypes = [vp, C.POINTER(stx_params), C.POINTER(stx_incidence), C.POINTER(stx_grads),
                                   C.c_float]
        L.stx_backward_sgd.argtypes = [vp, C.POINTER(stx_incidence), C.POINTER(stx_params), C.POINTER(stx_grads),
                                       C.c_float]
        L.stx_train_step.argtypes = [vp, C.POINTER(stx_batch), C.POINTER(stx_incidence), C.POINTER(stx_params),
                                     C.POINTER(stx_grads), C.c_float, vp, vp]
        L.stx_profile_kernel.argtypes = [vp, C.c_char_p, i32]
        L.stx_profile_every.argtypes = [vp, i32]
        L.stx_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
        L.stx_profile_dump.argtypes = [vp, C.c_char_p, C.c_size_t]
        L.stx_copy_f32.argtypes = [vp, vp, vp, i64]
        L.stx_read_sectors.argtypes = [vp, vp, i64, i32, i64, vp]
        L.stx_status_string.argtypes = [C.c_int]
        L.stx_status_string.restype = C.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().stx_status_string(status).decode()


def _check(call: str, status: int):
    if status != STX_OK:
        raise StxError(call, status)


def _ptr(t):
    return None if t is None else t.data_ptr()


def make_config(model, dist, n_ent, n_rel, dim, max_batch, max_neg, rel_dim=0, margin=1.0, reduce=STX_SUM,
                flags=0) -> stx_config:
    model = MODELS[model] if isinstance(model, str) else model
    dist = DISTS[dist] if isinstance(dist, str) else dist
    return stx_config(model, dist, reduce, dim, rel_dim or dim, n_ent, n_rel, margin, max_batch, max_neg, flags)


def stx_workspace_bytes(cfg: stx_config) -> int:
    n = C.c_size_t(0)
    _check("stx_workspace_bytes", lib().stx_workspace_bytes(C.byref(cfg), C.byref(n)))
    return n.value


class Context:
    """Owns the workspace tensor and the stx_ctx handle."""

    def __init__(self, cfg: stx_config, device="cuda:0", stream: torch.cuda.Stream | None = None):
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = stx_workspace_bytes(cfg)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        _check("stx_create", lib().stx_create(C.byref(cfg), self._ws_ptr, nbytes, self.stream.cuda_stream,
                                              C.byref(h)))
        self.handle = h

    @property
    def rows_max(self):
        return self.cfg.max_batch * (1 + self.cfg.max_neg)

    @property
    def cols_max(self):
        return min(3 * self.rows_max, self.cfg.n_ent + self.cfg.n_rel)

    @property
    def ld(self):
        return max(self.cfg.dim, self.cfg.rel_dim)

    def close(self):
        if self.handle:
            lib().stx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Incidence:
    """Device arrays of one stx_incidence, sized for the context's maxima."""

    def __init__(self, ctx: Context):
        dev, rows, nnz, cols = ctx.device, ctx.rows_max, 3 * ctx.rows_max, ctx.cols_max
        i32 = dict(dtype=torch.int32, device=dev)
        self.a_rowptr = torch.empty(rows + 1, **i32)
        self.a_colidx = torch.empty(nnz, **i32)
        self.a_vals = torch.empty(nnz, dtype=torch.float32, device=dev)
        self.at_touched_cols = torch.empty(cols, **i32)
        self.at_seg_ptr = torch.empty(cols + 1, **i32)
        self.at_row_idx = torch.empty(nnz, **i32)
        self.at_sign = torch.empty(nnz, dtype=torch.int8, device=dev)
        self.at_seg_id = torch.empty(nnz, **i32)
        self.at_packed = torch.empty(nnz, **i32)
        self.n_touched = torch.zeros(1, **i32)
        self.c = stx_incidence(0, 0, 0, 0, *(t.data_ptr() for t in (
            self.a_rowptr, self.a_colidx, self.a_vals, self.at_touched_cols, self.at_seg_ptr, self.at_row_idx,
            self.at_sign, self.at_seg_id, self.at_packed, self.n_touched)))

    @property
    def n_rows(self):
        return self.c.n_rows

    @property
    def nnz(self):
        return self.c.nnz


class Grads:
    def __init__(self, ctx: Context):
        f32 = dict(dtype=torch.float32, device=ctx.device)
        self.rows = torch.empty(ctx.cols_max, ctx.ld, **f32)
        self.w_rows = torch.empty(ctx.cols_max, ctx.ld, **f32) if ctx.cfg.model == STX_TRANSH else None
        self.proj = (torch.empty(ctx.cfg.n_rel, ctx.cfg.rel_dim, ctx.cfg.dim, **f32)
                     if ctx.cfg.model == STX_TRANSR else None)
        self.c = stx_grads(_ptr(self.rows), _ptr(self.w_rows), _ptr(self.proj))


class Params:
    def __init__(self, ent, rel=None, w=None, proj=None, rel_weight=None):
        self.ent, self.rel, self.w, self.proj, self.rel_weight = ent, rel, w, proj, rel_weight
        for t in (ent, rel, w, proj, rel_weight):
            assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous())
        self.c = stx_params(_ptr(ent), _ptr(rel), _ptr(w), _ptr(proj), _ptr(rel_weight))


def _i32dev(t):
    assert t is None or (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous())
    return _ptr(t)


def stx_sample_negatives(ctx: Context, h, r, t, k, seed, epoch, m_total, global_offset, neg_h, neg_t):
    m = h.numel()
    assert neg_h.numel() >= m * k and neg_t.numel() >= m * k
    _check("stx_sample_negatives",
           lib().stx_sample_negatives(ctx.handle, _i32dev(h), _i32dev(r), _i32dev(t), m, k, seed, epoch, m_total,
                                      global_offset, _i32dev(neg_h), _i32dev(neg_t)))


def stx_build_incidence(ctx: Context, h, r, t, neg_h, neg_t, k, inc: Incidence):
    b = h.numel()
    assert r.numel() == b and t.numel() == b
    assert k == 0 or (neg_h.numel() >= b * k and neg_t.numel() >= b * k)
    _check("stx_build_incidence",
           lib().stx_build_incidence(ctx.handle, _i32dev(h), _i32dev(r), _i32dev(t), _i32dev(neg_h),
                                     _i32dev(neg_t), b, k, C.byref(inc.c)))


def stx_check_indices(ctx: Context) -> int:
    n = C.c_int64(0)
    st = lib().stx_check_indices(ctx.handle, C.byref(n))
    if st not in (STX_OK, STX_ERR_INDEX_RANGE):
        raise StxError("stx_check_indices", st)
    return n.value


def stx_spmm(ctx: Context, inc: Incidence, p: Params, c_out):
    assert c_out.is_cuda and c_out.dtype == torch.float32 and c_out.is_contiguous()
    assert c_out.numel() >= inc.n_rows * ctx.cfg.dim
    _check("stx_spmm", lib().stx_spmm(ctx.handle, C.byref(inc.c), C.byref(p.c), c_out.data_ptr()))


def stx_spmm_semiring(ctx: Context, inc: Incidence, p: Params, kind: int, z_out):
    assert z_out.is_cuda and z_out.dtype == torch.float32 and z_out.is_contiguous()
    assert z_out.numel() >= inc.n_rows * ctx.cfg.dim
    _check("stx_spmm_semiring", lib().stx_spmm_semiring(ctx.handle, C.byref(inc.c), C.byref(p.c), kind,
                                                        z_out.data_ptr()))


def stx_spmm_semiring_t(ctx: Context, inc: Incidence, p: Params, kind: int, gz, work, g: Grads):
    for t in (gz, work):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert gz.numel() >= inc.n_rows * ctx.cfg.dim and work.numel() >= 3 * inc.n_rows * ctx.cfg.dim
    _check("stx_spmm_semiring_t", lib().stx_spmm_semiring_t(ctx.handle, C.byref(inc.c), C.byref(p.c), kind,
                                                            gz.data_ptr(), work.data_ptr(), C.byref(g.c)))


def stx_spmm_semiring_t_static(ctx: Context, inc: Incidence, p: Params, kind: int, gz, g: Grads):
    assert gz.is_cuda and gz.dtype == torch.float32 and gz.is_contiguous()
    assert gz.numel() >= inc.n_rows * ctx.cfg.dim
    _check("stx_spmm_semiring_t_static", lib().stx_spmm_semiring_t_static(ctx.handle, C.byref(inc.c), C.byref(p.c),
                                                                          kind, gz.data_ptr(), C.byref(g.c)))


def stx_rank_work_bytes(ctx: Context, nq: int) -> int:
    n = C.c_size_t(0)
    _check("stx_rank_work_bytes", lib().stx_rank_work_bytes(ctx.handle, nq, C.byref(n)))
    return n.value


def stx_rank(ctx: Context, p: Params, h, r, t, side: int, true_score, n_less, n_equal, work=None):
    """work: a uint8 device tensor of at least stx_rank_work_bytes(nq) + 256 bytes (TransR), else None."""
    nq = h.numel()
    assert r.numel() == nq and t.numel() == nq
    assert true_score.is_cuda and true_score.dtype == torch.float32 and true_score.numel() >= nq
    for c in (n_less, n_equal):
        assert c.is_cuda and c.dtype == torch.int32 and c.is_contiguous() and c.numel() >= nq
    wp, wb = None, 0
    if work is not None:
        assert work.is_cuda and work.dtype == torch.uint8 and work.is_contiguous()
        wp = (work.data_ptr() + 255) // 256 * 256
        wb = work.numel() - (wp - work.data_ptr())
    _check("stx_rank", lib().stx_rank(ctx.handle, C.byref(p.c), _i32dev(h), _i32dev(r), _i32dev(t), nq, side,
                                      true_score.data_ptr(), n_less.data_ptr(), n_equal.data_ptr(), wp, wb))


def stx_forward(ctx: Context, inc: Incidence, p: Params, scores, loss):
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.numel() >= inc.n_rows
    assert loss.is_cuda and loss.dtype == torch.float32 and loss.numel() >= 1
    _check("stx_forward", lib().stx_forward(ctx.handle, C.byref(inc.c), C.byref(p.c), scores.data_ptr(),
                                            loss.data_ptr()))


def stx_backward(ctx: Context, inc: Incidence, p: Params, g: Grads):
    _check("stx_backward", lib().stx_backward(ctx.handle, C.byref(inc.c), C.byref(p.c), C.byref(g.c)))


def stx_sgd_step(ctx: Context, p: Params, inc: Incidence, g: Grads, lr: float):
    _check("stx_sgd_step", lib().stx_sgd_step(ctx.handle, C.byref(p.c), C.byref(inc.c), C.byref(g.c), lr))


def stx_backward_sgd(ctx: Context, inc: Incidence, p: Params, g, lr: float):
    """g may be None for TransE / TorusE (no gradient rows are written)."""
    gp = C.byref(g.c) if g is not None else None
    _check("stx_backward_sgd", lib().stx_backward_sgd(ctx.handle, C.byref(inc.c), C.byref(p.c), gp, lr))


def make_batch(h, r, t, k, seed, epoch, m_total, global_offset, neg_h, neg_t, next_batch=None) -> "stx_batch":
    """Argument block of stx_train_step; the tensors (and next_batch, the block of the call that follows, if
    given) must stay alive while it is in use.  link_batches() chains a list of them."""
    b = h.numel()
    assert r.numel() == b and t.numel() == b
    assert k == 0 or (neg_h.numel() >= b * k and neg_t.numel() >= b * k)
    return stx_batch(_i32dev(h), _i32dev(r), _i32dev(t), b, k, seed, epoch, m_total, global_offset,
                     _i32dev(neg_h) if k else None, _i32dev(neg_t) if k else None,
                     C.addressof(next_batch) if next_batch is not None else None)


def link_batches(batches, cyclic=False):
    """Sets every block's `next` to the block after it (the last one's to the first when cyclic)."""
    for i, bt in enumerate(batches):
        nxt = batches[(i + 1) % len(batches)] if (cyclic or i + 1 < len(batches)) else None
        bt.next = C.addressof(nxt) if nxt is not None else None
    return batches


def stx_train_step(ctx: Context, batch, inc: Incidence, p: Params, g, lr: float, scores, loss):
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.numel() >= batch.b * (1 + batch.k)
    assert loss.is_cuda and loss.dtype == torch.float32 and loss.numel() >= 1
    gp = C.byref(g.c) if g is not None else None
    _check("stx_train_step", lib().stx_train_step(ctx.handle, C.byref(batch), C.byref(inc.c), C.byref(p.c), gp, lr,
                                                  scores.data_ptr(), loss.data_ptr()))


def stx_profile_kernel(ctx: Context, kernel_name, max_records: int):
    name = None if kernel_name is None else kernel_name.encode()
    _check("stx_profile_kernel", lib().stx_profile_kernel(ctx.handle, name, max_records))


def stx_profile_every(ctx: Context, every: int):
    _check("stx_profile_every", lib().stx_profile_every(ctx.handle, every))


def stx_profile_read(ctx: Context):
    """(mean microseconds per bracketed launch, number of launches recorded)."""
    avg, n = C.c_double(0), C.c_int32(0)
    _check("stx_profile_read", lib().stx_profile_read(ctx.handle, C.byref(avg), C.byref(n)))
    return avg.value, n.value


def stx_copy_f32(ctx: Context, dst, src):
    assert dst.numel() == src.numel() and dst.dtype == src.dtype == torch.float32
    _check("stx_copy_f32", lib().stx_copy_f32(ctx.handle, dst.data_ptr(), src.data_ptr(), src.numel()))


def stx_read_sectors(ctx: Context, src, n_slots: int, slot_bytes: int, n_reads: int, sink):
    assert src.is_cuda and src.numel() * src.element_size() >= n_slots * slot_bytes
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.numel() >= 16384
    _check("stx_read_sectors", lib().stx_read_sectors(ctx.handle, src.data_ptr(), n_slots, slot_bytes, n_reads,
                                                      sink.data_ptr()))


def stx_profile_dump(ctx: Context) -> dict:
    """{kernel name: (mean microseconds, launches)} of everything recorded since the last read."""
    buf = C.create_string_buffer(8192)
    _check("stx_profile_dump", lib().stx_profile_dump(ctx.handle, buf, len(buf)))
    out = {}
    for ln in buf.value.decode().splitlines():
        name, us, n = ln.split()
        out[name] = (float(us), int(n))
    return out
