"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def declared_symbols():
    text = "".join(p.read_text() for p in sorted((ROOT / "include").glob("*.h")))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(scd_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_mandated_calls():
    syms = declared_symbols()
    for name in ("scd_decompose", "scd_step", "scd_expand"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    from paper_2410_01799_amd import scd

    if not scd.LIB_PATH.exists():
        pytest.fail("libscd.so is not built: run __graft_entry__.build()")
    lib = ctypes.CDLL(str(scd.LIB_PATH))
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} declared in include/*.h but not exported"
    assert sorted(scd.EXPORTS) == declared_symbols()


def test_host_side_argument_checks_need_no_gpu():
    from paper_2410_01799_amd import scd

    L = scd.lib()
    assert L.scd_strerror(0) == b"ok"
    assert b"invalid" in L.scd_strerror(scd.EINVAL)
    dims = (ctypes.c_int64 * 2)(4, 4)
    h = ctypes.c_void_p()
    # null input, bad order, bad dtype, negative width: rejected before any device work
    assert L.scd_create(ctypes.byref(h), None, 0, 2, dims, 1, 0, None) == scd.EINVAL
    assert L.scd_create(ctypes.byref(h), ctypes.c_void_p(8), 0, 1, dims, 1, 0, None) == scd.EINVAL
    assert L.scd_create(ctypes.byref(h), ctypes.c_void_p(8), 7, 2, dims, 1, 0, None) == scd.EINVAL
    assert L.scd_create(ctypes.byref(h), ctypes.c_void_p(8), 0, 2, dims, -1, 0, None) == scd.EINVAL
    bad = (ctypes.c_int64 * 2)(4, 0)
    assert L.scd_create(ctypes.byref(h), ctypes.c_void_p(8), 0, 2, bad, 1, 0, None) == scd.EINVAL
    assert L.scd_run(None, 1) == scd.EINVAL
    assert L.scd_expand(None, None, 0, 2, dims, 0, None, None) == scd.EINVAL
    assert L.scd_pack(None, 0, 4, None, None) == scd.EINVAL
