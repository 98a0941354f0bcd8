"""The C-ABI library loads, exports every function include/adafuse.h declares, and
rejects bad arguments before touching a GPU (these run on a machine without one)."""
import ctypes as C
import os
import re

import pytest

import paper_2603_11873_amd as af
from paper_2603_11873_amd.binding import EXPORTS, MatrixDesc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, ERR_NULL, ERR_ARG, ERR_SHAPE, ERR_ALIGN, ERR_HIP = range(6)


@pytest.fixture(scope="module")
def L():
    return af.load_library()


def _desc(out=64, in_=64, ldw=None, wb=0x10000, ww=0x20000, a=0x30000, b=0x40000, reserved=0):
    return MatrixDesc(wb, ww, a, b, out, in_, in_ if ldw is None else ldw, reserved)


def _create(L, descs, E=8, r=8, k_max=2):
    arr = (MatrixDesc * max(len(descs), 1))(*descs)
    h = C.c_void_p()
    st = L.adafuse_create(arr, len(descs), E, r, k_max, C.byref(h))
    return st, h


def test_header_functions_are_exported(L):
    text = open(os.path.join(ROOT, "include", "adafuse.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(adafuse_[a-z_]+)\s*\(", text))
    assert declared == set(EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings(L):
    seen = {L.adafuse_status_string(s) for s in range(6)}
    assert len(seen) == 6 and all(seen)
    assert L.adafuse_status_string(99) == b"unknown status"


def test_create_rejects_bad_arguments(L):
    assert _create(L, [], 8, 8, 2)[0] == ERR_ARG
    arr = (MatrixDesc * 1)(_desc())
    assert L.adafuse_create(arr, 1, 8, 8, 2, None) == ERR_NULL
    h = C.c_void_p()
    assert L.adafuse_create(None, 1, 8, 8, 2, C.byref(h)) == ERR_NULL
    assert _create(L, [_desc(wb=0)])[0] == ERR_NULL
    assert _create(L, [_desc(b=0)])[0] == ERR_NULL
    assert _create(L, [_desc()], E=0)[0] == ERR_ARG
    assert _create(L, [_desc()], E=65)[0] == ERR_ARG
    assert _create(L, [_desc()], r=7)[0] == ERR_ARG
    assert _create(L, [_desc()], r=256)[0] == ERR_ARG
    assert _create(L, [_desc()], k_max=0)[0] == ERR_ARG
    assert _create(L, [_desc()], E=4, k_max=5)[0] == ERR_ARG
    assert _create(L, [_desc()], E=16, k_max=9)[0] == ERR_ARG
    assert _create(L, [_desc(reserved=1)])[0] == ERR_ARG
    assert _create(L, [_desc(ww=0x10000), _desc()])[0] == ERR_ARG  # in-place and out-of-place mixed
    assert _create(L, [_desc(ww=0x10000)], E=16, k_max=5)[0] == ERR_ARG   # in place: 2 k_max terms at most 8
    assert _create(L, [_desc(out=0)])[0] == ERR_SHAPE
    assert _create(L, [_desc(in_=4)])[0] == ERR_SHAPE
    assert _create(L, [_desc(in_=100)])[0] == ERR_SHAPE
    assert _create(L, [_desc(in_=64, ldw=56)])[0] == ERR_SHAPE
    assert _create(L, [_desc(in_=64, ldw=68)])[0] == ERR_SHAPE
    assert _create(L, [_desc(in_=64, ldw=(1 << 24) + 8)])[0] == ERR_SHAPE   # beyond the 32-bit offsets inside a tile
    assert _create(L, [_desc(in_=(1 << 22) + 8, ldw=(1 << 22) + 8)])[0] == ERR_SHAPE
    assert _create(L, [_desc(wb=0x10008)])[0] == ERR_ALIGN
    assert _create(L, [_desc(a=0x30002)])[0] == ERR_ALIGN
    # second descriptor bad, first good
    assert _create(L, [_desc(), _desc(out=-3)])[0] == ERR_SHAPE


@pytest.mark.parametrize("inplace", [False, True])
def test_valid_create_needs_a_device_or_succeeds(L, inplace):
    st, h = _create(L, [_desc(ww=0x10000 if inplace else 0x20000)])
    assert st in (OK, ERR_HIP)       # no GPU here -> ERR_HIP, never a crash; tables only, no launch
    if st == OK:
        assert L.adafuse_destroy(h) == OK
    else:
        assert not h.value
    assert L.adafuse_destroy(None) == OK


def test_pregate_rejects_bad_arguments(L):
    hid, wr, idx, g = 0x10000, 0x20000, 0x30000, 0x40000

    def call(hidden=hid, w=wr, T=4, d=64, E=8, k=2, norm=0, idx_=idx, gates=g):
        return L.adafuse_pregate(hidden, w, T, d, E, k, norm, idx_, gates, None, None)

    assert call(hidden=None) == ERR_NULL
    assert call(idx_=None) == ERR_NULL
    assert call(gates=None) == ERR_NULL
    assert call(T=-1) == ERR_ARG
    assert call(k=0) == ERR_ARG
    assert call(k=9, E=16) == ERR_ARG
    assert call(k=3, E=2) == ERR_ARG
    assert call(E=65) == ERR_ARG
    assert call(norm=2) == ERR_ARG
    assert call(d=60) == ERR_SHAPE
    assert call(hidden=hid + 2) == ERR_ALIGN
    assert call(T=0) == OK            # nothing to do, nothing launched


def test_switch_and_misc_reject_null_context(L):
    assert L.adafuse_fused_switch(None, None, None, None, None, 2, 2.0, 0, None) == ERR_NULL
    assert L.adafuse_switch_per_matrix(None, None, None, None, None, 2, 2.0, 0, None) == ERR_NULL
    assert L.adafuse_forward_merged(None, None, None, None) == ERR_NULL
    assert L.adafuse_forward_dynamic(None, None, None, 2, 2.0, None, None, None, None) == ERR_NULL
    assert L.adafuse_set_option(None, 0, 1) == ERR_NULL
    assert L.adafuse_get_info(None, None) == ERR_NULL
