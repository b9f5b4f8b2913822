"""Host-side checks that need no GPU: the library loads, exports every declared symbol, and rejects
bad configurations before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2502_16949_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = "".join(open(os.path.join(ROOT, "include", f)).read() for f in ("stx.h", "stx_measure.h"))
    return sorted(set(re.findall(r"\b(stx_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared()
    assert set(B.EXPORTS) == set(names), (names, B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    assert B.status_string(B.STX_OK) == "ok"
    seen = {B.status_string(i) for i in range(9)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert B.status_string(99) == "unknown status"


@pytest.mark.parametrize("kw,status", [
    (dict(), B.STX_OK),
    (dict(dim=30), B.STX_ERR_BAD_ARG),                 # not a multiple of 4
    (dict(dim=2048), B.STX_ERR_BAD_ARG),
    (dict(model=9), B.STX_ERR_BAD_ARG),
    (dict(dist=-1), B.STX_ERR_BAD_ARG),
    (dict(n_ent=0), B.STX_ERR_BAD_ARG),
    (dict(n_ent=2**31), B.STX_ERR_BAD_ARG),
    (dict(max_batch=0), B.STX_ERR_BAD_ARG),
    (dict(max_batch=2**27, max_neg=1), B.STX_ERR_BAD_ARG),
    (dict(margin=-1.0), B.STX_ERR_BAD_ARG),
    (dict(flags=8), B.STX_ERR_BAD_ARG),
])
def test_config_validation(kw, status):
    base = dict(model="transe", dist="l1", n_ent=100, n_rel=5, dim=32, max_batch=64, max_neg=1)
    base.update(kw)
    cfg = B.make_config(**base)
    n = C.c_size_t(0)
    assert B.lib().stx_workspace_bytes(C.byref(cfg), C.byref(n)) == status
    if status == B.STX_OK:
        assert n.value > 0 and n.value % 256 == 0


def test_null_arguments_are_rejected_without_a_device():
    lib = B.lib()
    cfg = B.make_config("transe", "l1", 100, 5, 32, 64, 1)
    assert lib.stx_workspace_bytes(C.byref(cfg), None) == B.STX_ERR_NULL
    assert lib.stx_workspace_bytes(None, C.byref(C.c_size_t())) == B.STX_ERR_NULL
    h = C.c_void_p()
    assert lib.stx_create(C.byref(cfg), None, 1 << 30, None, C.byref(h)) == B.STX_ERR_NULL
    assert lib.stx_create(C.byref(cfg), 256, 16, None, C.byref(h)) == B.STX_ERR_WORKSPACE   # too small
    assert lib.stx_create(C.byref(cfg), 257, 1 << 30, None, C.byref(h)) == B.STX_ERR_WORKSPACE  # misaligned
    assert lib.stx_destroy(None) == B.STX_ERR_NULL
    assert lib.stx_forward(None, None, None, None, None) == B.STX_ERR_NULL


def test_workspace_grows_with_the_batch():
    a = B.stx_workspace_bytes(B.make_config("transe", "l1", 15000, 1350, 128, 32768, 1))
    b = B.stx_workspace_bytes(B.make_config("transe", "l1", 15000, 1350, 128, 65536, 1))
    assert b > a >= 65536 * 128 * 4
