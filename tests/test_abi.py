"""The C-ABI library loads and exports every symbol that include/gvq.h declares, and its
host-side argument checks work without a GPU (no kernel is launched here)."""
import ctypes as C
import os
import re

import pytest

from paper_1811_03617_amd import gvq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "gvq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gvq_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_codec_calls():
    names = _declared()
    for n in ("gvq_fit_basis", "gvq_compress", "gvq_aggregate", "gvq_decompress"):
        assert n in names


def test_every_declared_symbol_is_exported():
    L = gvq.lib()
    for name in _declared():
        assert hasattr(L, name), name


def test_strerror_and_option_checks():
    assert gvq.strerror(gvq.OK) == "ok"
    for s in (gvq.EINVAL, gvq.EALIGN, gvq.ENOTFIT, gvq.EHIP, gvq.ENOMEM, gvq.ENONFINITE, gvq.ENOCONV):
        assert gvq.strerror(s) and gvq.strerror(s) != "unknown status"
    assert gvq.strerror(-99) == "unknown status"
    assert gvq.lib().gvq_set_option(99, 1) == gvq.EINVAL
    assert gvq.lib().gvq_set_option(0, 0) == gvq.OK
    assert gvq.lib().gvq_set_option(5, 4097) == gvq.EINVAL
    assert gvq.lib().gvq_set_option(5, -1) == gvq.EINVAL
    assert gvq.lib().gvq_set_option(5, 0) == gvq.OK


@pytest.mark.parametrize("M,d,k,nb,offs", [
    (0, 16, 4, 1, None),        # no elements
    (100, 1, 1, 1, None),       # d too small
    (100, 1025, 4, 1, None),    # d too large
    (100, 16, 0, 1, None),      # k too small
    (100, 16, 17, 1, None),     # k > d
    (100, 16, 4, 2, None),      # several bases need offsets
    (16 * 70000, 16, 4, 65536, list(range(65537))),   # more bases than a handle takes
    (160, 16, 4, 2, [0, 5, 9]),   # offsets do not end at S = 10
    (160, 16, 4, 2, [0, 5, 5]),   # not increasing
    (160, 16, 4, 2, [1, 5, 10]),  # does not start at 0
])
def test_create_rejects_bad_arguments_before_touching_the_device(M, d, k, nb, offs):
    h = C.c_void_p()
    arr = None if offs is None else (C.c_int64 * len(offs))(*offs)
    assert gvq.lib().gvq_basis_create(C.byref(h), M, d, k, nb, arr, gvq.F32) == gvq.EINVAL
    assert not h.value
    assert gvq.lib().gvq_basis_create(None, 100, 16, 4, 1, None, gvq.F32) == gvq.EINVAL
    assert gvq.lib().gvq_basis_create(C.byref(h), 100, 16, 4, 1, None, 7) == gvq.EINVAL


def test_null_handle_is_rejected():
    L = gvq.lib()
    assert L.gvq_num_slices(None) == gvq.EINVAL
    assert L.gvq_compress(None, None, 1, None, None) == gvq.EINVAL
    assert L.gvq_decompress(None, None, None, 0, None) == gvq.EINVAL
    assert L.gvq_aggregate(None, None, 1, None, None) == gvq.EINVAL
    assert L.gvq_fit_basis(None, None, 1, None) == gvq.EINVAL
    assert L.gvq_basis_destroy(None) == gvq.OK
