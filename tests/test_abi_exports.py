"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before touching any device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "msx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(msx_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def L():
    import paper_2504_09014_amd as msx
    return msx.lib()


def test_every_declared_symbol_is_exported(L):
    import paper_2504_09014_amd as msx
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n
    assert sorted(msx.EXPORTS) == names


def test_strerror_and_version(L):
    assert b"gfx950" in L.msx_version()
    assert L.msx_strerror(0) == b"ok"
    for code in range(-7, 0):
        assert L.msx_strerror(code) not in (b"ok", b"unknown error")
    assert L.msx_strerror(-99) == b"unknown error"


def test_argument_errors_need_no_device(L):
    fake = C.c_void_p(0x1000)      # aligned, never dereferenced: every call below fails first
    odd = C.c_void_p(0x1004)
    ARG, UNSUP = -1, -2
    assert L.msx_allreduce(fake, 16, 7, 0, 8, None) == ARG          # dtype
    assert L.msx_allreduce(fake, 16, 0, 3, 8, None) == UNSUP        # op (sum, max, min exist)
    assert L.msx_allreduce(fake, 16, 0, 0, 0, None) == ARG          # nranks
    assert L.msx_allreduce(fake, 16, 0, 0, 9, None) == ARG
    assert L.msx_allreduce(None, 16, 0, 0, 8, None) == ARG
    assert L.msx_allreduce(odd, 16, 0, 0, 8, None) == ARG           # alignment
    assert L.msx_allreduce(fake, 0, 0, 0, 8, None) == 0             # empty is a no-op
    assert L.msx_reducescatter(fake, 12, 0, 0, 8, None) == ARG      # count % nranks
    assert L.msx_alltoall(fake, 12, 1, 0, 8, None) == ARG
    assert L.msx_reducescatter(fake, 0, 0, 0, 8, None) == 0
    assert L.msx_allgather(None, 4, 0, 0, 8, None) == ARG
    tbl = (C.c_void_p * 8)(*[0x1000 + 0x100 * i for i in range(8)])
    bad = (C.c_void_p * 8)(*[0x1000 + 0x100 * i for i in range(7)], 0)
    pp = C.POINTER(C.c_void_p)
    assert L.msx_allreduce_ex(C.cast(bad, pp), C.cast(tbl, pp), None, 16, 0, 0, 8, 0, None) == ARG
    assert L.msx_allreduce_ex(C.cast(tbl, pp), C.cast(tbl, pp), None, 16, 0, 0, 8, 11, None) == ARG  # algo
    assert L.msx_allreduce_ex(C.cast(tbl, pp), C.cast(tbl, pp), None, 0, 0, 0, 8, 0, None) == 0
    assert L.msx_alltoall_ex(C.cast(tbl, pp), C.cast(tbl, pp), 64, 0, 8, None) == ARG                 # overlap
    assert L.msx_moe_dispatch(C.cast(tbl, pp), C.cast(tbl, pp), 4, 7, 8, 256, 1, 8, C.cast(tbl, pp), None,
                              fake, 16, None, None) == ARG                                             # row % 16
    assert L.msx_moe_dispatch(C.cast(tbl, pp), C.cast(tbl, pp), 70000, 8, 8, 256, 1, 8, C.cast(tbl, pp), None,
                              fake, 16, None, None) == UNSUP
    # handles: unknown ones are refused before any device is touched
    assert L.msx_ctx_use(fake) == ARG
    assert L.msx_ctx_use(None) == 0
    assert L.msx_ctx_destroy(fake) == ARG
    assert L.msx_ctx_set_max_blocks(fake, 8) == ARG
    assert L.msx_run(None, None) == ARG
    assert L.msx_release(None) == 0
    assert L.msx_release(fake) == ARG
    assert L.msx_moe_plan_destroy(fake) == ARG
    h = C.c_void_p()
    assert L.msx_ctx_create(9, 0, C.byref(h)) == ARG
    assert L.msx_ctx_create(8, 100, C.byref(h)) == ARG                                                # LL size
    assert L.msx_prepare_allreduce(C.cast(tbl, pp), C.cast(tbl, pp), None, 16, 0, 0, 8, 0, None) == ARG
    assert L.msx_prim_pingpong(10, 1, 0, 0, fake, None) == ARG
    assert L.msx_prim_barrier(1, 9, 1, None, None) == ARG
    assert L.msx_set_option(b"no_such_key", b"1") == ARG
    assert L.msx_set_option(b"hb_unroll", b"3") == ARG
    assert L.msx_set_option(b"algo", b"ring") == ARG


def test_options_roundtrip_without_device(L):
    import paper_2504_09014_amd as msx
    for key, val in [("algo", "2pa_ll"), ("hb_unroll", "4"), ("spin_limit", "12345"), ("drop_rank", "3"),
                     ("chaos", "7"), ("hb_barriers", "0")]:
        old = msx.get_option(key)
        msx.set_option(key, val)
        assert msx.get_option(key) == val
        msx.set_option(key, old)
        assert msx.get_option(key) == old


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_09014_amd")
    pat = re.compile(r"import\s+oracle|from\s+oracle|from\s+\.\.?\s*oracle|msx_oracle|orc_[a-z]")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not pat.search(text), (dirpath, f)
