"""Pins for the CPU oracle's values: things the paper and mathematics fix, independent of the oracle.

Every check compares the interpreter (oracle.access_pattern / oracle.programs) and the C loops
(oracle.brute) with something that is neither: pure-Python loops typed here from the paper's
equations, closed forms, special cases with a textbook answer, and numpy library routines.
"""

import itertools
import math

import numpy as np
import pytest
import torch

from oracle import access_pattern as ap
from oracle import brute, numerics
from oracle import programs as pg


def rng(seed):
    return np.random.default_rng(seed)


# -- pure-Python loops from the paper's equations (tiny sizes only) ------------

def conv2d_loops(A, W, S, P=(0, 0)):
    """out[n,o,x,y] = sum_{dx,dy,c} A[n,c,S0*x+dx,S1*y+dy] * W[o,c,dx,dy]  (Sec. 5.1), zero padding P."""
    N, C, H, Wd = A.shape
    O, _, Kh, Kw = W.shape
    Ho = (H + 2 * P[0] - Kh) // S[0] + 1
    Wo = (Wd + 2 * P[1] - Kw) // S[1] + 1
    out = [[[[0 for _ in range(Wo)] for _ in range(Ho)] for _ in range(O)] for _ in range(N)]
    for n, o, x, y in itertools.product(range(N), range(O), range(Ho), range(Wo)):
        acc = 0
        for dx, dy, c in itertools.product(range(Kh), range(Kw), range(C)):
            h, w = S[0] * x + dx - P[0], S[1] * y + dy - P[1]
            if 0 <= h < H and 0 <= w < Wd:
                acc += A[n, c, h, w].item() * W[o, c, dx, dy].item()
        out[n][o][x][y] = acc
    return np.array(out)


def maxpool_loops(A, K, S):
    """out[n,c,x,y] = max_{dx,dy} A[n,c,S0*x+dx,S1*y+dy]  (Sec. 5.1)."""
    N, C, H, Wd = A.shape
    Ho, Wo = (H - K[0]) // S[0] + 1, (Wd - K[1]) // S[1] + 1
    out = np.empty((N, C, Ho, Wo), dtype=A.dtype)
    for n, c, x, y in itertools.product(range(N), range(C), range(Ho), range(Wo)):
        out[n, c, x, y] = max(A[n, c, S[0] * x + dx, S[1] * y + dy]
                              for dx in range(K[0]) for dy in range(K[1]))
    return out


CONV_CASES = [
    # N C H W  O Kh Kw  S      P
    (1, 3, 8, 8, 4, 3, 3, (1, 1), (0, 0)),       # the tiny configuration's shape
    (2, 2, 7, 9, 3, 3, 2, (2, 1), (0, 0)),       # non-square everything, mixed strides
    (1, 1, 6, 5, 1, 2, 3, (1, 2), (1, 2)),       # C = O = 1, asymmetric padding sizes
    (2, 3, 5, 5, 2, 5, 5, (1, 1), (0, 0)),       # window == full extent
    (1, 2, 9, 9, 2, 3, 3, (3, 3), (1, 1)),       # stride 3 with padding
    (1, 3, 8, 6, 2, 1, 1, (2, 2), (0, 0)),       # 1x1 stride 2 (projection shortcut)
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d_three_ways_int(case):
    N, C, H, Wd, O, Kh, Kw, S, P = case
    r = rng(hash(case) % 1000)
    A = r.integers(-8, 9, (N, C, H, Wd))
    W = r.integers(-8, 9, (O, C, Kh, Kw))
    want = conv2d_loops(A, W, S, P)
    got_direct = pg.conv2d(ap.tensor(A), ap.tensor(W), S, P).materialize()
    got_im2col = pg.conv2d_im2col(ap.tensor(A), ap.tensor(W), S, P).materialize()
    got_c = brute.conv2d(A, W, S, P)
    assert got_direct.dtype == np.int64
    np.testing.assert_array_equal(got_direct, want)
    np.testing.assert_array_equal(got_im2col, want)          # Fig. 2a == Fig. 5
    np.testing.assert_array_equal(got_c, want)


def test_conv2d_float_against_loops():
    r = rng(5)
    A = r.standard_normal((1, 2, 6, 7))
    W = r.standard_normal((3, 2, 3, 2))
    want = conv2d_loops(A, W, (1, 2), (1, 0))
    np.testing.assert_allclose(pg.conv2d(ap.tensor(A), ap.tensor(W), (1, 2), (1, 0)).materialize(),
                               want, rtol=0, atol=1e-12)
    np.testing.assert_allclose(brute.conv2d(A, W, (1, 2), (1, 0)), want, rtol=0, atol=1e-12)


def test_conv2d_delta_kernel_is_shifted_strided_channel():
    """A one-hot weight W[o, c0, dx0, dy0] = 1 makes out[n,o,x,y] = A[n,c0,S0*x+dx0,S1*y+dy0]."""
    r = rng(7)
    A = r.integers(-100, 100, (2, 3, 9, 8))
    S = (2, 1)
    for (c0, dx0, dy0) in [(0, 0, 0), (2, 1, 2), (1, 2, 0)]:
        W = np.zeros((1, 3, 3, 3), dtype=np.int64)
        W[0, c0, dx0, dy0] = 1
        Ho, Wo = (9 - 3) // 2 + 1, (8 - 3) // 1 + 1
        want = A[:, c0, dx0:dx0 + S[0] * Ho:S[0], dy0:dy0 + S[1] * Wo:S[1]][:, None]
        np.testing.assert_array_equal(pg.conv2d(ap.tensor(A), ap.tensor(W), S).materialize(), want)
        np.testing.assert_array_equal(brute.conv2d(A, W, S), want)


def test_conv2d_all_ones_counts_window_elements():
    A = np.ones((1, 4, 6, 6), dtype=np.int64)
    W = np.ones((2, 4, 3, 3), dtype=np.int64)
    assert (pg.conv2d(ap.tensor(A), ap.tensor(W), (1, 1)).materialize() == 36).all()
    padded = pg.conv2d(ap.tensor(A), ap.tensor(W), (1, 1), (1, 1)).materialize()
    assert padded.shape == (1, 2, 6, 6)
    assert padded[0, 0, 0, 0] == 16 and padded[0, 0, 0, 3] == 24 and padded[0, 0, 3, 3] == 36
    np.testing.assert_array_equal(brute.conv2d(A, W, (1, 1), (1, 1)), padded)


def test_conv2d_1x1_is_matmul_over_channels():
    r = rng(11)
    A = r.standard_normal((2, 5, 4, 3))
    W = r.standard_normal((6, 5, 1, 1))
    want = np.einsum("nchw,oc->nohw", A, W[:, :, 0, 0])
    np.testing.assert_allclose(pg.conv2d(ap.tensor(A), ap.tensor(W), (1, 1)).materialize(), want,
                               atol=1e-12)
    np.testing.assert_allclose(brute.conv2d(A, W, (1, 1)), want, atol=1e-12)


def test_windows_element_rule_and_cartprod_order():
    """windows: out[a,p,q] = A[a, p*s+q]; cartProd puts the first input at tuple slot 0."""
    A = np.arange(2 * 10).reshape(2, 10)
    win = ap.windows(ap.access(ap.tensor(A), 1), (4,), (3,)).materialize()
    assert win.shape == (2, 3, 4)
    for a, p, q in itertools.product(range(2), range(3), range(4)):
        assert win[a, p, q] == A[a, p * 3 + q]
    X = np.array([[1, 2, 3], [4, 5, 6]])
    Y = np.array([[10, 20, 30], [40, 50, 60], [70, 80, 90], [11, 12, 13]])
    cp = ap.cart_prod(ap.access(ap.tensor(X), 1), ap.access(ap.tensor(Y), 1)).materialize()
    assert cp.shape == (2, 4, 2, 3)
    for i, j in itertools.product(range(2), range(4)):
        np.testing.assert_array_equal(cp[i, j, 0], X[i])
        np.testing.assert_array_equal(cp[i, j, 1], Y[j])


def test_matmul_against_loops_library_and_identity():
    r = rng(13)
    P = r.integers(-9, 9, (5, 7))
    Q = r.integers(-9, 9, (7, 3))
    want = np.array([[sum(P[i, k].item() * Q[k, j].item() for k in range(7)) for j in range(3)]
                     for i in range(5)])                       # R_ij = sum_k P_ik Q_kj, Sec. 3.1
    np.testing.assert_array_equal(pg.matmul(ap.tensor(P), ap.tensor(Q)).materialize(), want)
    np.testing.assert_array_equal(brute.matmul(P, Q), want)
    np.testing.assert_array_equal(want, P @ Q)
    Pf, Qf = r.standard_normal((33, 17)), r.standard_normal((17, 29))
    np.testing.assert_allclose(pg.matmul(ap.tensor(Pf), ap.tensor(Qf)).materialize(), Pf @ Qf, atol=1e-12)
    np.testing.assert_allclose(brute.matmul(Pf, Qf), Pf @ Qf, atol=1e-12)
    np.testing.assert_array_equal(pg.matmul(ap.tensor(P), ap.tensor(np.eye(7, dtype=np.int64))).materialize(), P)


def test_dotprod_commutes_and_cartesian_dot_is_nt_product():
    r = rng(17)
    a0, a1 = r.standard_normal((6, 11)), r.standard_normal((4, 11))
    x, y = ap.access(ap.tensor(a0), 1), ap.access(ap.tensor(a1), 1)
    lhs = pg.cartesian_dot(x, y).materialize()
    np.testing.assert_allclose(lhs, a0 @ a1.T, atol=1e-12)
    np.testing.assert_allclose(pg.cartesian_dot(y, x).materialize(), lhs.T, atol=1e-12)   # dotProd(P,Q)=dotProd(Q,P)


@pytest.mark.parametrize("shape,K,S", [((2, 3, 7, 8), (2, 2), (2, 2)), ((1, 2, 9, 7), (3, 3), (2, 2)),
                                       ((1, 1, 5, 6), (2, 3), (1, 2)), ((2, 2, 4, 4), (4, 4), (1, 1))])
def test_maxpool_against_loops(shape, K, S):
    A = rng(19).integers(-50, 50, shape)
    want = maxpool_loops(A, K, S)
    np.testing.assert_array_equal(pg.max_pool2d(ap.tensor(A), K, S).materialize(), want)
    np.testing.assert_array_equal(brute.max_pool2d(A, K, S), want)


def test_maxpool_closed_forms():
    A = rng(23).standard_normal((2, 3, 5, 6))
    full = pg.max_pool2d(ap.tensor(A), (5, 6), (1, 1)).materialize()       # window == extent -> global max
    np.testing.assert_array_equal(full[:, :, 0, 0], A.max(axis=(2, 3)))
    ramp = np.arange(8 * 9, dtype=np.float64).reshape(1, 1, 8, 9)           # increasing -> last element of window
    got = pg.max_pool2d(ap.tensor(ramp), (3, 2), (2, 3)).materialize()
    for x, y in itertools.product(range(got.shape[2]), range(got.shape[3])):
        assert got[0, 0, x, y] == (2 * x + 2) * 9 + (3 * y + 1)
    # padding with the lowest value never wins; padded output keeps real maxima at the border
    padded = pg.max_pool2d(ap.tensor(A), (3, 3), (2, 2), (1, 1), -np.inf).materialize()
    assert padded.shape == (2, 3, 3, 3)
    assert padded[0, 0, 0, 0] == A[0, 0, 0:2, 0:2].max()
    np.testing.assert_array_equal(brute.max_pool2d(A, (3, 3), (2, 2), (1, 1), -np.inf), padded)


def test_reduce_sum_pins():
    ones = np.ones((3, 4, 5, 6), dtype=np.int64)
    assert (ap.compute(ap.reduceSum, ap.access(ap.tensor(ones), 2)).materialize() == 30).all()
    r = rng(29)
    a, b = r.standard_normal((4, 5)), r.standard_normal((4, 5))
    x, y = ap.access(ap.tensor(a), 2), ap.access(ap.tensor(b), 2)
    np.testing.assert_array_equal(pg.add(x, y).materialize(), a + b)       # reduceSum(pair a b) == a + b
    X = r.integers(-5, 5, (7, 13))
    np.testing.assert_array_equal(brute.row_reduce(X, False), X.sum(axis=1))
    np.testing.assert_array_equal(brute.row_reduce(X, True), X.max(axis=1))
    np.testing.assert_array_equal(ap.compute(ap.reduceMax, ap.access(ap.tensor(X), 1)).materialize(), X.max(axis=1))
    # the real-valued instance of the same loops: closed forms, then random rows against an
    # exactly rounded sum (math.fsum) and numpy's max
    ones_f = np.ones((5, 1024), dtype=np.float64)
    np.testing.assert_array_equal(brute.row_reduce(ones_f, False), np.full(5, 1024.0))
    ramp = np.tile(np.arange(1.0, 101.0), (3, 1)) * np.array([[1.0], [-1.0], [0.5]])
    np.testing.assert_array_equal(brute.row_reduce(ramp, False), [5050.0, -5050.0, 2525.0])
    np.testing.assert_array_equal(brute.row_reduce(ramp, True), [100.0, -1.0, 50.0])
    F = r.standard_normal((9, 257)) * 10.0 ** r.integers(-3, 4, (9, 257))
    exact = np.array([math.fsum(row) for row in F])
    got_f = brute.row_reduce(F, False)
    assert np.abs(got_f - exact).max() <= 257 * 2.0 ** -52 * np.abs(F).sum(axis=1).max()
    np.testing.assert_array_equal(brute.row_reduce(F, True), F.max(axis=1))
    neg = -np.abs(F) - 1.0                                    # a max that must not start from zero
    np.testing.assert_array_equal(brute.row_reduce(neg, True), neg.max(axis=1))
    assert brute.row_reduce(np.zeros((4, 0)), False).tolist() == [0.0] * 4   # empty sum
    with pytest.raises(ValueError):
        brute.row_reduce(np.zeros((4, 0)), True)              # max of nothing


def test_transformer_values():
    A = np.arange(2 * 3 * 4).reshape(2, 3, 4)
    t = ap.transpose(ap.access(ap.tensor(A), 1), (2, 0, 1)).materialize()
    np.testing.assert_array_equal(t, np.transpose(A, (2, 0, 1)))
    np.testing.assert_array_equal(ap.slice_(ap.tensor(A), 2, 1, 3).materialize(), A[:, :, 1:3])
    np.testing.assert_array_equal(ap.flatten(ap.access(ap.tensor(A), 1)).materialize(), A.reshape(2, 12))
    np.testing.assert_array_equal(ap.reshape(ap.access(ap.tensor(A), 1), (2,), (4, 3)).materialize(),
                                  A.reshape(2, 4, 3))
    B = A + 100
    p = ap.pair(ap.access(ap.tensor(A), 1), ap.access(ap.tensor(B), 1)).materialize()
    np.testing.assert_array_equal(p, np.stack([A, B], axis=1))
    c = ap.concat(ap.tensor(A), ap.tensor(B[:, :2]), 1).materialize()
    np.testing.assert_array_equal(c, np.concatenate([A, B[:, :2]], axis=1))
    pd = ap.pad(ap.tensor(A), 1, 1, 2, -7).materialize()
    np.testing.assert_array_equal(pd, np.pad(A, ((0, 0), (1, 2), (0, 0)), constant_values=-7))
    sq = ap.squeeze(ap.tensor(A[:, :1]), 1).materialize()
    np.testing.assert_array_equal(sq, A[:, 0])


def test_extension_operators():
    x = np.array([[-1.5, 0.0, 2.0]])
    np.testing.assert_array_equal(ap.compute(ap.relu, ap.access(ap.tensor(x), 2)).materialize(), [[0, 0, 2.0]])
    np.testing.assert_array_equal(ap.compute(ap.scale(0.5), ap.access(ap.tensor(x), 2)).materialize(),
                                  [[-0.75, 0, 1.0]])


def test_sampled_positions_equal_full_evaluation():
    r = rng(31)
    A, W = r.integers(-8, 9, (2, 3, 9, 9)), r.integers(-8, 9, (5, 3, 3, 3))
    prog = pg.conv2d(ap.tensor(A), ap.tensor(W), (2, 2), (1, 1))
    full = prog.materialize()
    pts = np.stack([r.integers(0, s, 50) for s in full.shape], axis=1)
    np.testing.assert_array_equal(prog.gather_points(pts), full[tuple(pts.T)])
    assert prog.at(1, 4, 2, 3) == full[1, 4, 2, 3]


def test_depthwise_program_against_block_diagonal_convolution_and_closed_forms():
    """The depth-wise program (slice / Fig. 2a / concat) equals an ordinary convolution whose
    weights are zero off the channel diagonal, equals explicit loops, and a one-hot filter tap
    copies the shifted, strided channel."""
    r = rng(61)
    n, c, h, w, kh, kw = 2, 5, 9, 8, 3, 2
    x = r.integers(-9, 10, (n, c, h, w))
    f = r.integers(-9, 10, (c, 1, kh, kw))
    for stride, pad in (((1, 1), (0, 0)), ((2, 1), (1, 1)), ((2, 3), (2, 0))):
        got = pg.depthwise_conv2d(ap.tensor(x), ap.tensor(f), stride, pad).materialize()
        full = np.zeros((c, c, kh, kw), dtype=np.int64)
        for ch in range(c):
            full[ch, ch] = f[ch, 0]
        np.testing.assert_array_equal(got, brute.conv2d(x, full, stride, pad))
        xp = np.pad(x, ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
        ho, wo = (h + 2 * pad[0] - kh) // stride[0] + 1, (w + 2 * pad[1] - kw) // stride[1] + 1
        assert got.shape == (n, c, ho, wo)
        for (i, ch, y, xx) in [(0, 0, 0, 0), (1, 4, ho - 1, wo - 1), (1, 2, ho // 2, 1)]:
            want = sum(int(xp[i, ch, y * stride[0] + a, xx * stride[1] + b]) * int(f[ch, 0, a, b])
                       for a in range(kh) for b in range(kw))
            assert got[i, ch, y, xx] == want
    tap = np.zeros((c, 1, kh, kw), dtype=np.int64)
    tap[:, 0, 2, 1] = np.arange(1, c + 1)                 # channel ch: (ch + 1) * x[.., y*2 + 2, x + 1]
    got = pg.depthwise_conv2d(ap.tensor(x), ap.tensor(tap), (2, 1), (0, 0)).materialize()
    want = x[:, :, 2::2, 1:][:, :, :got.shape[2], :got.shape[3]] * np.arange(1, c + 1)[None, :, None, None]
    np.testing.assert_array_equal(got, want)


# -- storage-type conversions ------------------------------------------------------

def test_bf16_conversions_against_torch():
    r = rng(37)
    x = np.concatenate([r.standard_normal(5000).astype(np.float32) * 10.0 ** r.integers(-20, 20, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, np.inf, -np.inf,
                                  1e-40, 65280.0], dtype=np.float32)]).astype(np.float32)
    bits = numerics.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(bits, want.view(torch.int16).numpy().view(np.uint16))
    np.testing.assert_array_equal(numerics.bf16_bits_to_f64(bits), want.to(torch.float64).numpy())
    # ties to even, by hand: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1; 1 + 3*2^-8 -> 1 + 2^-6
    assert numerics.bf16_bits_to_f64(numerics.f32_to_bf16_bits(np.float32(1 + 2 ** -8))) == 1.0
    assert numerics.bf16_bits_to_f64(numerics.f32_to_bf16_bits(np.float32(1 + 3 * 2 ** -8))) == 1 + 2 ** -6


def test_e4m3_decode_against_torch_and_by_hand():
    """Every one of the 256 bit patterns against torch's float8_e4m3fn -> float32 conversion, and the
    values the OCP format fixes by definition."""
    bits = np.arange(256, dtype=np.uint8)
    got = numerics.e4m3_bits_to_f64(bits)
    want = torch.from_numpy(bits.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    by_hand = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x3C: 1.5,
               0x40: 2.0, 0x7E: 448.0, 0xC0: -2.0, 0xB8: -1.0, 0xFE: -448.0}
    for b, v in by_hand.items():
        assert got[b] == v, hex(b)
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.signbit(got[0x80]) and got[0x80] == 0.0
    assert (np.diff(got[:0x7F]) > 0).all()          # positive patterns are ordered like their bits
    np.testing.assert_array_equal(got[0x80:0xFF], -got[0x00:0x7F])


def test_i32_check_refuses_overflow():
    assert numerics.to_i32_checked(np.array([2 ** 31 - 1, -2 ** 31])).dtype == np.int32
    with pytest.raises(OverflowError):
        numerics.to_i32_checked(np.array([2 ** 31]))
