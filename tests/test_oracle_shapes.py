"""Shape rules of Table 1 / Table 2 and the shape annotations of the paper's listings."""

import numpy as np
import pytest

from oracle import access_pattern as ap
from oracle import programs as pg


def T(*shape):
    return ap.tensor(np.zeros(shape))


def parse_dims(text, env):
    text = text.strip()
    if not text:
        return ()
    return tuple(int(eval(tok, {}, env)) for tok in text.split(","))


def load_golden(golden_dir, listing):
    rows = []
    with open(golden_dir + "/listing_shapes.txt") as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, node, acc, cmp_ = [p.strip() for p in line.split("|")]
            if name == listing:
                rows.append((node, acc, cmp_))
    assert rows
    return rows


# -- Table 1, one test per row ---------------------------------------------

def test_access_resplits():
    t = T(5, 7)
    assert ap.access(t, 1).ap_shape == ((5,), (7,))          # Sec. 4.1 example: (m,n) -> ((m),(n))
    assert ap.access(t, 0).ap_shape == ((), (5, 7))
    assert ap.access(t, 2).ap_shape == ((5, 7), ())
    with pytest.raises(ValueError):
        ap.access(t, 3)


def test_transpose_shape_and_split():
    q = ap.access(T(6, 4), 1)                                # Sec. 4.2 example: Q (N,O) -> ((O),(N))
    assert ap.transpose(q, (1, 0)).ap_shape == ((4,), (6,))
    a = ap.access(T(2, 3, 4, 5), 4)
    assert ap.transpose(a, (0, 3, 1, 2)).ap_shape == ((2, 5, 3, 4), ())
    with pytest.raises(ValueError):
        ap.transpose(q, (0, 0))


def test_cartprod_shape():
    a = ap.access(T(3, 4, 7, 2), 2)
    b = ap.access(T(5, 7, 2), 1)
    assert ap.cart_prod(a, b).ap_shape == ((3, 4, 5), (2, 7, 2))
    with pytest.raises(ValueError):
        ap.cart_prod(a, ap.access(T(5, 7, 3), 1))


@pytest.mark.parametrize("b,w,s,expect", [(8, 3, 1, 6), (30, 3, 2, 14), (7, 7, 1, 1), (10, 3, 3, 3),
                                          (9, 2, 2, 4), (230, 7, 2, 112)])
def test_windows_dim_formula(b, w, s, expect):
    assert ap.windows_out_dim(b, w, s) == expect
    assert ap.windows_out_dim(b, w, s) == (b - w) // s + 1   # same thing for integers b >= w


def test_windows_shape():
    a = ap.access(T(2, 3, 8, 9), 1)
    assert ap.windows(a, (3, 3, 2), (1, 1, 2)).ap_shape == ((2, 1, 6, 4), (3, 3, 2))
    with pytest.raises(ValueError):
        ap.windows(a, (3, 3), (1, 1))
    with pytest.raises(ValueError):
        ap.windows(a, (4, 3, 3), (1, 1, 1))


def test_slice_squeeze_flatten_reshape_pair_concat_shapes():
    a = ap.access(T(4, 6, 8), 1)
    assert ap.slice_(a, 1, 2, 5).ap_shape == ((4,), (3, 8))
    assert ap.squeeze(ap.access(T(4, 1, 8), 2), 1).ap_shape == ((4,), (8,))
    assert ap.squeeze(ap.access(T(4, 8, 1), 1), 2).ap_shape == ((4,), (8,))
    assert ap.squeeze(ap.access(T(4, 1, 8), 1), 1).ap_shape == ((4,), (8,))     # first compute dim
    with pytest.raises(ValueError):
        ap.squeeze(a, 1)
    assert ap.flatten(ap.access(T(2, 3, 4, 5), 2)).ap_shape == ((6,), (20,))
    assert ap.flatten(ap.access(T(2, 3), 2)).ap_shape == ((6,), ())
    assert ap.reshape(ap.access(T(6, 20), 1), (2, 3), (4, 5)).ap_shape == ((2, 3), (4, 5))
    with pytest.raises(ValueError):
        ap.reshape(ap.access(T(6, 20), 1), (4, 3), (2, 5))
    assert ap.pair(a, a).ap_shape == ((4,), (2, 6, 8))
    with pytest.raises(ValueError):
        ap.pair(a, ap.access(T(4, 6, 8), 2))
    assert ap.concat(a, ap.access(T(4, 2, 8), 1), 1).ap_shape == ((4,), (8, 8))
    with pytest.raises(ValueError):
        ap.concat(a, ap.access(T(4, 2, 7), 1), 1)


def test_compute_keeps_access_dims():
    a = ap.access(T(3, 5, 2, 4), 2)
    for op in (ap.reduceSum, ap.reduceMax, ap.dotProd):
        assert ap.compute(op, a).ap_shape == ((3, 5), ())


# -- listings -----------------------------------------------------------------

@pytest.mark.parametrize("env", [
    dict(N=2, C=3, H=8, W=9, O=4, Kh=3, Kw=2, Sh=1, Sw=2),
    dict(N=1, C=5, H=11, W=11, O=2, Kh=5, Kw=5, Sh=3, Sw=3),
])
def test_fig2a_fig5_shape_traces(golden_dir, env):
    e = dict(env)
    e["Ho"] = ap.windows_out_dim(e["H"], e["Kh"], e["Sh"])
    e["Wo"] = ap.windows_out_dim(e["W"], e["Kw"], e["Sw"])
    act = ap.access(T(e["N"], e["C"], e["H"], e["W"]), 1)
    wts = ap.access(T(e["O"], e["C"], e["Kh"], e["Kw"]), 1)
    win = ap.windows(act, (e["C"], e["Kh"], e["Kw"]), (1, e["Sh"], e["Sw"]))
    cp = ap.cart_prod(win, wts)
    dp = ap.compute(ap.dotProd, cp)
    sq = ap.squeeze(dp, 1)
    tr = ap.transpose(sq, (0, 3, 1, 2))
    got = [act, wts, win, cp, dp, sq, tr]
    for node, (name, acc, cmp_) in zip(got, load_golden(golden_dir, "fig2a")):
        assert node.ap_shape == (parse_dims(acc, e), parse_dims(cmp_, e)), name
    assert pg.conv2d(T(e["N"], e["C"], e["H"], e["W"]), T(e["O"], e["C"], e["Kh"], e["Kw"]),
                     (e["Sh"], e["Sw"])).ap_shape == tr.ap_shape

    fw, fk = ap.flatten(win), ap.flatten(wts)
    dp5 = ap.compute(ap.dotProd, ap.cart_prod(fw, fk))
    rs = ap.reshape(dp5, (e["N"], 1, e["Ho"], e["Wo"], e["O"]), ())
    for node, (name, acc, cmp_) in zip([fw, fk, dp5, rs], load_golden(golden_dir, "fig5")):
        assert node.ap_shape == (parse_dims(acc, e), parse_dims(cmp_, e)), name


def test_fig2b_shape_trace(golden_dir):
    e = dict(M=5, N=7, O=3)
    act = ap.access(T(e["M"], e["N"]), 1)
    wts = ap.access(T(e["N"], e["O"]), 1)
    tr = ap.transpose(wts, (1, 0))
    cp = ap.cart_prod(act, tr)
    dp = ap.compute(ap.dotProd, cp)
    for node, (name, acc, cmp_) in zip([act, wts, tr, cp, dp], load_golden(golden_dir, "fig2b")):
        assert node.ap_shape == (parse_dims(acc, e), parse_dims(cmp_, e)), name


def test_fig2c_shape_trace(golden_dir):
    e = dict(N=2, C=3, H=9, W=8, Kh=3, Kw=2, Sh=2, Sw=2)
    e["Ho"] = ap.windows_out_dim(e["H"], e["Kh"], e["Sh"])
    e["Wo"] = ap.windows_out_dim(e["W"], e["Kw"], e["Sw"])
    act = ap.access(T(e["N"], e["C"], e["H"], e["W"]), 2)
    win = ap.windows(act, (e["Kh"], e["Kw"]), (e["Sh"], e["Sw"]))
    mx = ap.compute(ap.reduceMax, win)
    for node, (name, acc, cmp_) in zip([act, win, mx], load_golden(golden_dir, "fig2c")):
        assert node.ap_shape == (parse_dims(acc, e), parse_dims(cmp_, e)), name


def test_fig7_shape_trace_and_block_count(golden_dir):
    a = ap.access(T(32, 32), 1)
    w = ap.access(T(32, 32), 1)
    a_blk = ap.slice_(ap.slice_(a, 0, 0, 16), 1, 0, 16)
    w_blk = ap.transpose(ap.slice_(ap.slice_(w, 0, 0, 16), 1, 0, 16), (1, 0))
    cp = ap.cart_prod(a_blk, w_blk)
    dp = ap.compute(ap.dotProd, cp)
    pr = ap.pair(dp, dp)
    rs = ap.compute(ap.reduceSum, pr)
    c1 = ap.concat(rs, rs, 1)
    c0 = ap.concat(c1, c1, 0)
    for node, (name, acc, cmp_) in zip([a_blk, w_blk, cp, dp, pr, rs, c1, c0],
                                       load_golden(golden_dir, "fig7")):
        assert node.ap_shape == (parse_dims(acc, {}), parse_dims(cmp_, {})), name
    prog, count = pg.blocked_matmul(T(32, 32), T(32, 32), 16)
    assert count == 8                      # Sec. 5.4: eight separate 16x16 matMuls
    assert prog.ap_shape == ((32, 32), ())
