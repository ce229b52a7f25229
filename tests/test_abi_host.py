"""The C ABI without a GPU: the library loads, exports what the header declares, and rejects bad
arguments on the host before anything is launched."""

import ctypes
import os
import re

import pytest

from paper_2105_09377_amd import binding as gs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000   # aligned, non-null, never dereferenced: validation fails first in every test


def ap(shape, n_access, dtype=gs.GS_BF16, data=FAKE):
    a = gs.gs_ap()
    a.data, a.dtype, a.rank, a.n_access, a.reserved = data, dtype, len(shape), n_access, 0
    for i, s in enumerate(shape):
        a.shape[i] = s
    return a


def i64(*v):
    return (ctypes.c_int64 * len(v))(*v)


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "glenside.h")) as fh:
        header = fh.read()
    declared = set(re.findall(r"\b(glenside_\w+)\s*\(", header))
    assert declared == set(gs.EXPORTS)
    lib = gs.lib()
    for name in declared:
        # without declared argument types ctypes would pass pointers (streams, workspaces) as 32-bit ints
        assert getattr(lib, name).argtypes is not None, name


def test_status_strings():
    assert gs.status_string(gs.GS_OK) == "ok"
    assert "shape" in gs.status_string(gs.GS_ERR_SHAPE)
    assert "unknown" in gs.status_string(99)


def test_struct_layout_matches_header():
    assert ctypes.sizeof(gs.gs_ap) == 8 + 4 * 4 + 8 * gs.GS_MAX_RANK
    assert gs.gs_ap.shape.offset == 24


@pytest.mark.parametrize("shape,na,window,stride,lo,hi,want", [
    ((2, 3, 8, 9), 1, (3, 3, 2), (1, 1, 2), None, None, ((2, 1, 6, 4, 3, 3, 2), 4)),
    ((32, 64, 56, 56), 1, (64, 3, 3), (1, 1, 1), (0, 1, 1), (0, 1, 1), ((32, 1, 56, 56, 64, 3, 3), 4)),
    ((64, 64, 112, 112), 2, (3, 3), (2, 2), (1, 1), (1, 1), ((64, 64, 56, 56, 3, 3), 4)),
    ((5, 10), 1, (4,), (3,), None, None, ((5, 3, 4), 2)),
])
def test_windows_shape_rule(shape, na, window, stride, lo, hi, want):
    assert gs.windows_out_shape(shape, na, window, stride, lo, hi) == want


def test_windows_shape_errors():
    with pytest.raises(gs.GlensideError) as e:
        gs.windows_out_shape((2, 8), 1, (9,), (1,))          # window larger than the dimension
    assert e.value.status == gs.GS_ERR_SHAPE
    with pytest.raises(gs.GlensideError) as e:
        gs.windows_out_shape((2, 8), 2, (3,), (1,))          # no compute dimension to window
    assert e.value.status == gs.GS_ERR_RANK
    with pytest.raises(gs.GlensideError) as e:
        gs.windows_out_shape((2, 8), 1, (3,), (0,))          # stride 0
    assert e.value.status == gs.GS_ERR_SHAPE


def test_cartesian_dot_validation():
    L = gs.lib()
    call = lambda a0, a1, out, act=0: L.glenside_cartesian_dot(ctypes.byref(a0), ctypes.byref(a1),
                                                               ctypes.byref(out), act, None, 0, None)
    good0, good1 = ap((4, 16), 1), ap((8, 16), 1)
    assert call(good0, ap((8, 15), 1), ap((4, 8), 2, gs.GS_F32)) == gs.GS_ERR_SHAPE      # compute dims differ
    assert call(good0, good1, ap((4, 9), 2, gs.GS_F32)) == gs.GS_ERR_SHAPE               # wrong result shape
    assert call(good0, good1, ap((4, 8), 1, gs.GS_F32)) == gs.GS_ERR_RANK                # result must be all-access
    assert call(good0, good1, ap((4, 8), 2, gs.GS_I32)) == gs.GS_ERR_DTYPE               # bf16 -> i32
    assert call(good0, ap((8, 16), 1, gs.GS_I8), ap((4, 8), 2, gs.GS_F32)) == gs.GS_ERR_DTYPE
    assert call(good0, good1, ap((4, 8), 2, gs.GS_F32), act=7) == gs.GS_ERR_UNSUPPORTED
    assert call(ap((4, 16), 1, data=0), good1, ap((4, 8), 2, gs.GS_F32)) == gs.GS_ERR_NULL
    assert call(ap((4, 16), 1, data=FAKE + 2), good1, ap((4, 8), 2, gs.GS_F32)) == gs.GS_ERR_UNSUPPORTED
    assert L.glenside_cartesian_dot(None, ctypes.byref(good1), ctypes.byref(good1), 0, None, 0, None) == gs.GS_ERR_NULL
    bad_rank = ap((4, 16), 1)
    bad_rank.rank = 9
    assert call(bad_rank, good1, ap((4, 8), 2, gs.GS_F32)) == gs.GS_ERR_RANK


def test_conv_validation_and_workspace_queries():
    L = gs.lib()
    x, w = ap((2, 3, 8, 8), 1, gs.GS_I8), ap((4, 3, 3, 3), 1, gs.GS_I8)
    st, pd = i64(1, 1), i64(0, 0)
    out = ap((2, 4, 6, 6), 4, gs.GS_I32)
    for fn in (L.glenside_conv2d_direct, L.glenside_conv2d_im2col):
        call = lambda x_, w_, out_, ws=FAKE, nbytes=1 << 30, res=None: fn(
            ctypes.byref(x_), ctypes.byref(w_), st, pd, res, 0, ctypes.byref(out_), ws, nbytes, None)
        assert call(x, ap((4, 2, 3, 3), 1, gs.GS_I8), out) == gs.GS_ERR_SHAPE       # channel mismatch
        assert call(x, w, ap((2, 4, 6, 5), 4, gs.GS_I32)) == gs.GS_ERR_SHAPE         # wrong H'/W'
        assert call(x, w, ap((2, 4, 6, 6), 4, gs.GS_F32)) == gs.GS_ERR_DTYPE         # i8 must give i32
        assert call(ap((2, 3, 8, 8), 2, gs.GS_I8), w, out) == gs.GS_ERR_RANK         # activations are (access x 1)
        assert call(x, ap((4, 3, 9, 3), 1, gs.GS_I8), out) == gs.GS_ERR_SHAPE        # window taller than the image
        assert call(x, w, out, ws=None) == gs.GS_ERR_WORKSPACE
        assert call(x, w, out, nbytes=8) == gs.GS_ERR_WORKSPACE
        assert call(x, w, out, res=ctypes.byref(ap((2, 4, 6, 6), 4, gs.GS_F32))) == gs.GS_ERR_DTYPE
    d = L.glenside_conv2d_direct_workspace(ctypes.byref(x), ctypes.byref(w), st, pd)
    m = L.glenside_conv2d_im2col_workspace(ctypes.byref(x), ctypes.byref(w), st, pd)
    assert d >= 4 * 9 * 32                      # repacked weights, channels padded to a 32-byte step
    assert m >= 2 * 36 * 32                     # 72 windows of 27 int8, rows padded to 32 bytes
    assert L.glenside_conv2d_direct_workspace(ctypes.byref(x), ctypes.byref(ap((4, 2, 3, 3), 1, gs.GS_I8)), st, pd) == 0


def test_reduce_and_pair_validation():
    L = gs.lib()
    red = lambda a, op, scale, out: L.glenside_reduce(ctypes.byref(a), op, ctypes.c_float(scale), ctypes.byref(out), None)
    x = ap((4, 5, 7, 7), 2)
    assert red(x, gs.GS_SUM, 1.0, ap((4, 6), 2)) == gs.GS_ERR_SHAPE
    assert red(x, gs.GS_SUM, 1.0, ap((4, 5, 1), 3)) == gs.GS_ERR_RANK
    assert red(x, 5, 1.0, ap((4, 5), 2)) == gs.GS_ERR_UNSUPPORTED
    assert red(x, gs.GS_MAX, 0.5, ap((4, 5), 2)) == gs.GS_ERR_UNSUPPORTED            # scale only for float sums
    assert red(ap((4, 5, 7, 7), 2, gs.GS_I8), gs.GS_SUM, 1.0, ap((4, 5), 2, gs.GS_I8)) == gs.GS_ERR_DTYPE
    assert red(ap((4, 0), 1), gs.GS_MAX, 1.0, ap((4,), 1)) == gs.GS_ERR_SHAPE        # max of an empty element
    pr = lambda a, b, out: L.glenside_pair_reduce(ctypes.byref(a), ctypes.byref(b), 0, 0, ctypes.byref(out), None)
    y = ap((4, 5), 2, gs.GS_F32)
    assert pr(y, ap((4, 6), 2, gs.GS_F32), y) == gs.GS_ERR_SHAPE
    assert pr(y, ap((4, 5), 2, gs.GS_BF16), y) == gs.GS_ERR_DTYPE
    assert pr(ap((4, 5), 1, gs.GS_F32), ap((4, 5), 1, gs.GS_F32), y) == gs.GS_ERR_RANK   # compute dims would be folded


def test_transformer_validation():
    """Table 1 shape rules of transpose / slice / concat / pair (and the pad extension)."""
    L = gs.lib()
    x = ap((4, 5, 6), 1)
    other = 0x20000
    tr = lambda a, perm, out: L.glenside_transpose(ctypes.byref(a), i64(*perm), ctypes.byref(out), None)
    assert tr(x, (0, 0, 1), ap((4, 4, 5), 1, data=other)) == gs.GS_ERR_SHAPE          # not a permutation
    assert tr(x, (2, 0, 1), ap((6, 4, 6), 1, data=other)) == gs.GS_ERR_SHAPE          # result is (6, 4, 5)
    assert tr(x, (2, 0, 1), ap((6, 4, 5), 2, data=other)) == gs.GS_ERR_RANK           # the split stays at 1
    assert tr(x, (2, 0, 1), ap((6, 4, 5), 1, gs.GS_F32, data=other)) == gs.GS_ERR_DTYPE
    assert tr(x, (2, 0, 1), ap((6, 4, 5), 1)) == gs.GS_ERR_UNSUPPORTED                 # in place
    assert L.glenside_transpose(ctypes.byref(x), None, ctypes.byref(ap((6, 4, 5), 1, data=other)), None) == gs.GS_ERR_NULL
    sl = lambda a, d, lo, hi, out: L.glenside_slice(ctypes.byref(a), d, lo, hi, ctypes.byref(out), None)
    assert sl(x, 3, 0, 1, ap((4, 5, 6), 1, data=other)) == gs.GS_ERR_RANK
    assert sl(x, 1, 2, 6, ap((4, 4, 6), 1, data=other)) == gs.GS_ERR_SHAPE            # hi past the extent
    assert sl(x, 1, 3, 2, ap((4, 0, 6), 1, data=other)) == gs.GS_ERR_SHAPE            # lo > hi
    assert sl(x, 1, 1, 3, ap((4, 3, 6), 1, data=other)) == gs.GS_ERR_SHAPE            # result is (4, 2, 6)
    cc = lambda a, b, d, out: L.glenside_concat(ctypes.byref(a), ctypes.byref(b), d, ctypes.byref(out), None)
    assert cc(x, ap((4, 5, 7), 1), 1, ap((4, 10, 6), 1, data=other)) == gs.GS_ERR_SHAPE   # other dims differ
    assert cc(x, ap((4, 5, 6), 2), 1, ap((4, 10, 6), 1, data=other)) == gs.GS_ERR_RANK    # access splits differ
    assert cc(x, ap((4, 2, 6), 1), 1, ap((4, 8, 6), 1, data=other)) == gs.GS_ERR_SHAPE    # result is (4, 7, 6)
    assert cc(x, ap((4, 2, 6), 1, gs.GS_F32), 1, ap((4, 7, 6), 1, data=other)) == gs.GS_ERR_DTYPE
    pd = lambda a, d, lo, hi, mode, out: L.glenside_pad(ctypes.byref(a), d, lo, hi, mode, ctypes.byref(out), None)
    assert pd(x, 2, -1, 0, gs.GS_PAD_ZERO, ap((4, 5, 5), 1, data=other)) == gs.GS_ERR_SHAPE
    assert pd(x, 2, 1, 2, 7, ap((4, 5, 9), 1, data=other)) == gs.GS_ERR_UNSUPPORTED
    assert pd(x, 2, 1, 2, gs.GS_PAD_ZERO, ap((4, 5, 8), 1, data=other)) == gs.GS_ERR_SHAPE
    pr = lambda a, b, out: L.glenside_pair(ctypes.byref(a), ctypes.byref(b), ctypes.byref(out), None)
    assert pr(x, ap((4, 5, 7), 1), ap((4, 2, 5, 6), 1, data=other)) == gs.GS_ERR_SHAPE
    assert pr(x, x, ap((4, 5, 2, 6), 1, data=other)) == gs.GS_ERR_SHAPE               # the 2 leads the compute dims
    assert pr(x, x, ap((4, 2, 5, 6), 2, data=other)) == gs.GS_ERR_RANK
    full = ap((1,) * 8, 4)
    assert pr(full, full, ap((1,) * 8, 4, data=other)) == gs.GS_ERR_RANK              # rank 9 does not exist


def test_results_that_overlap_an_input_are_refused():
    """Partial overlaps, not only equal pointers: x is 4*5*6 bfloat16 = 240 bytes at FAKE."""
    L = gs.lib()
    x = ap((4, 5, 6), 1)
    for delta in (16, 224, -16):                              # the result starts inside / ends inside x
        at = FAKE + delta
        assert L.glenside_transpose(ctypes.byref(x), i64(2, 0, 1), ctypes.byref(ap((6, 4, 5), 1, data=at)), None) == gs.GS_ERR_UNSUPPORTED
        assert L.glenside_slice(ctypes.byref(x), 1, 1, 3, ctypes.byref(ap((4, 2, 6), 1, data=at)), None) == gs.GS_ERR_UNSUPPORTED
        assert L.glenside_pad(ctypes.byref(x), 2, 1, 1, gs.GS_PAD_ZERO, ctypes.byref(ap((4, 5, 8), 1, data=at)), None) == gs.GS_ERR_UNSUPPORTED
        b = ap((4, 2, 6), 1, data=0x40000)
        assert L.glenside_concat(ctypes.byref(x), ctypes.byref(b), 1, ctypes.byref(ap((4, 7, 6), 1, data=at)), None) == gs.GS_ERR_UNSUPPORTED
        assert L.glenside_concat(ctypes.byref(b), ctypes.byref(x), 1, ctypes.byref(ap((4, 7, 6), 1, data=at)), None) == gs.GS_ERR_UNSUPPORTED
        y = ap((4, 5, 6), 1, data=0x40000)
        assert L.glenside_pair(ctypes.byref(y), ctypes.byref(x), ctypes.byref(ap((4, 2, 5, 6), 1, data=at)), None) == gs.GS_ERR_UNSUPPORTED


def test_depthwise_validation():
    L = gs.lib()
    x, w = ap((2, 8, 14, 14), 1), ap((8, 3, 3), 1)
    other = 0x80000
    dw = lambda a, f, s, p, out, act=gs.GS_ACT_NONE: L.glenside_depthwise_conv2d(
        ctypes.byref(a), ctypes.byref(f), i64(*s), i64(*p), act, ctypes.byref(out), None)
    good = ap((2, 8, 14, 14), 4, data=other)
    assert dw(x, ap((7, 3, 3), 1), (1, 1), (1, 1), good) == gs.GS_ERR_SHAPE            # one filter per channel
    assert dw(x, ap((8, 1, 3, 3), 1), (1, 1), (1, 1), good) == gs.GS_ERR_RANK
    assert dw(x, w, (1, 1), (1, 1), ap((2, 8, 12, 12), 4, data=other)) == gs.GS_ERR_SHAPE
    assert dw(x, w, (2, 2), (1, 1), ap((2, 8, 7, 7), 1, data=other)) == gs.GS_ERR_RANK  # the result is all access dims
    assert dw(x, w, (0, 1), (1, 1), good) == gs.GS_ERR_SHAPE
    assert dw(x, w, (1, 1), (3, 3), ap((2, 8, 18, 18), 4, data=other)) == gs.GS_ERR_UNSUPPORTED   # padding >= window
    assert dw(x, w, (1, 1), (1, 1), ap((2, 8, 14, 14), 4, gs.GS_I32, data=other)) == gs.GS_ERR_DTYPE
    assert dw(x, ap((8, 3, 3), 1, gs.GS_I8), (1, 1), (1, 1), good) == gs.GS_ERR_DTYPE
    assert dw(ap((2, 8, 14, 14), 1, gs.GS_F32), ap((8, 3, 3), 1, gs.GS_F32), (1, 1), (1, 1),
              ap((2, 8, 14, 14), 4, gs.GS_F32, data=other)) == gs.GS_ERR_DTYPE
    assert dw(x, w, (1, 1), (1, 1), good, act=9) == gs.GS_ERR_UNSUPPORTED
    assert dw(x, w, (1, 1), (1, 1), ap((2, 8, 14, 14), 4, data=FAKE + 64)) == gs.GS_ERR_UNSUPPORTED   # overlaps x
    assert dw(ap((2, 8, 2, 14), 1), w, (1, 1), (0, 0), ap((2, 8, 0, 12), 4, data=other)) == gs.GS_ERR_SHAPE  # window taller than the image


def test_blocked_dot_validation():
    L = gs.lib()
    call = lambda a0, a1, tm, tn, tk, out: L.glenside_cartesian_dot_blocked(
        ctypes.byref(a0), ctypes.byref(a1), tm, tn, tk, ctypes.byref(out), None)
    a0, a1 = ap((64, 128), 1), ap((32, 128), 1)
    out = ap((64, 32), 2, gs.GS_F32, data=0x20000)
    assert call(a0, a1, 0, 16, 16, out) == gs.GS_ERR_SHAPE                         # tile sizes start at 1
    assert call(a0, ap((32, 64), 1), 16, 16, 16, out) == gs.GS_ERR_SHAPE           # compute shapes differ
    assert call(a0, a1, 16, 16, 16, ap((64, 32), 2, gs.GS_BF16, data=0x20000)) == gs.GS_ERR_DTYPE   # folds need 32 bits
    assert call(a0, a1, 16, 16, 16, ap((64, 33), 2, gs.GS_F32, data=0x20000)) == gs.GS_ERR_SHAPE
    assert call(ap((4, 16, 128), 2), a1, 16, 16, 16, out) == gs.GS_ERR_RANK        # stated for matrices
    big0, big1 = ap((4096, 4096), 1), ap((4096, 4096), 1)
    assert call(big0, big1, 16, 16, 16, ap((4096, 4096), 2, gs.GS_F32, data=0x20000)) == gs.GS_ERR_UNSUPPORTED


def test_windows_reduce_validation():
    L = gs.lib()
    call = lambda a, win, st, out, op=gs.GS_MAX: L.glenside_windows_reduce(
        ctypes.byref(a), win, st, None, None, op, ctypes.c_float(1.0), ctypes.byref(out), None)
    x = ap((2, 3, 8, 8), 2)
    assert call(x, i64(2, 2), i64(2, 2), ap((2, 3, 4, 3), 4)) == gs.GS_ERR_SHAPE
    assert call(x, i64(9, 2), i64(2, 2), ap((2, 3, 4, 4), 4)) == gs.GS_ERR_SHAPE
    assert call(x, i64(2, 2), i64(2, 2), ap((2, 3, 4, 4), 4, gs.GS_I32)) == gs.GS_ERR_DTYPE
