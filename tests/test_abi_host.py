"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, sizes workspaces, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2510_16415_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mecefo.h")).read()
    names = sorted(set(re.findall(r"\b(mecefo_[a-z_0-9]+)\s*\(", hdr)))
    assert {"mecefo_ffn_fwd_recompute", "mecefo_ffn_bwd_exact", "mecefo_ffn_bwd_lowrank",
            "mecefo_block_bwd_skip", "mecefo_workspace_bytes", "mecefo_last_error"} <= set(names)
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert B.mecefo_version().startswith("mecefo")


def test_workspace_bytes_grows_with_the_problem():
    small = B.mecefo_workspace_bytes(B.make_desc(256, 256, 688, B.F32), 32, 32, 32)
    big = B.mecefo_workspace_bytes(B.make_desc(8192, 4096, 11008, B.BF16), 1024, 1024, 1024)
    assert 0 < small < big
    # three [b x f] activations dominate at the 7B shape
    assert big >= 3 * 8192 * 11008 * 2


def _err(fn, *a):
    with pytest.raises(B.MecefoError) as e:
        fn(*a)
    return e.value


def test_descriptor_validation():
    e = _err(B.mecefo_workspace_bytes, B.make_desc(16, 64, 100, B.BF16), 8, 8, 8)   # ld_act_f=100 not %8
    assert e.status == B.ERR_INVALID_ARG and "multiple of 8" in str(e)
    e = _err(B.mecefo_workspace_bytes, B.make_desc(16, 60, 104, B.BF16), 8, 8, 8)   # d % 8 != 0
    assert e.status in (B.ERR_UNSUPPORTED, B.ERR_INVALID_ARG)
    e = _err(B.mecefo_workspace_bytes, B.make_desc(16, 64, 104, B.BF16, ld_act_d=32), 8, 8, 8)
    assert e.status == B.ERR_INVALID_ARG
    e = _err(B.mecefo_workspace_bytes, B.make_desc(-1, 64, 104, B.F32), 8, 8, 8)
    assert e.status == B.ERR_INVALID_ARG
    e = _err(B.mecefo_workspace_bytes, B.make_desc(16, 64, 104, B.F32, grad_dtype=B.BF16), 8, 8, 8)
    assert e.status == B.ERR_UNSUPPORTED
    e = _err(B.mecefo_workspace_bytes, B.make_desc(1 << 20, 4096, 11008, B.BF16), 8, 8, 8)   # > 2 GiB tensor
    assert e.status == B.ERR_UNSUPPORTED


def test_null_and_rank_validation_happens_before_any_launch():
    lib = B.lib()
    d = B.make_desc(16, 64, 104, B.BF16)
    P = B.Proj(0x1000, 8, 8)
    fake = C.c_void_p(0x10000)
    st = lib.mecefo_block_bwd_skip(C.byref(d), None, fake, fake, fake, fake, fake, P, P, P, 0,
                                   fake, fake, fake, fake, fake, 0, fake, 1 << 30, None)
    assert st == B.ERR_INVALID_ARG and "H is NULL" in B.mecefo_last_error()
    bad = B.Proj(0x1000, 65, 72)   # rank above the projected dimension d = 64
    st = lib.mecefo_block_bwd_skip(C.byref(d), fake, fake, fake, fake, fake, fake, bad, P, P, 0,
                                   fake, fake, fake, fake, fake, 0, fake, 1 << 30, None)
    assert st == B.ERR_INVALID_ARG and "rank" in B.mecefo_last_error()
    st = lib.mecefo_block_bwd_skip(C.byref(d), fake, fake, fake, fake, fake, fake, P, P, P, 0,
                                   fake, fake, fake, fake, fake, 0, fake, 16, None)
    assert st == B.ERR_WORKSPACE_TOO_SMALL
    mis = C.c_void_p(0x10002)
    st = lib.mecefo_ffn_bwd_lowrank(C.byref(d), mis, fake, fake, fake, fake, P, P, P, 0,
                                    fake, fake, fake, fake, 0, fake, 1 << 30, None)
    assert st == B.ERR_INVALID_ARG and "aligned" in B.mecefo_last_error()
    st = lib.mecefo_ffn_bwd_exact(C.byref(d), fake, fake, fake, fake, fake, fake, None,
                                  fake, fake, fake, fake, 0, fake, 1 << 30, None)
    assert st == B.ERR_INVALID_ARG and "both" in B.mecefo_last_error()
    st = lib.mecefo_block_bwd_skip(C.byref(d), fake, fake, fake, fake, fake, fake, P, P, P, 7,
                                   fake, fake, fake, fake, fake, 0, fake, 1 << 30, None)
    assert st == B.ERR_INVALID_ARG and "side" in B.mecefo_last_error()
