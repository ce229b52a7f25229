"""The paper's rewrites are equalities: both sides of each rule must evaluate identically.

Covers the systolic-array rewrite (Sec. 5.2), the three im2col rewrites (Sec. 5.3) and the five
blocking rewrites (Sec. 5.4), plus the blocked 32x32 matMul of Fig. 7.  Integer inputs make every
comparison exact.
"""

import numpy as np
import pytest

from oracle import access_pattern as ap
from oracle import programs as pg


def ints(seed, *shape):
    return np.random.default_rng(seed).integers(-9, 10, shape)


def same(x: ap.AP, y: ap.AP):
    assert x.ap_shape == y.ap_shape
    np.testing.assert_array_equal(x.materialize(), y.materialize())


def test_systolic_array_rewrite():
    a0 = ap.access(ap.tensor(ints(1, 7, 5)), 1)       # ((batch),(rows))
    a1 = ap.access(ap.tensor(ints(2, 3, 5)), 1)       # ((cols),(rows))
    lhs = ap.compute(ap.dotProd, ap.cart_prod(a0, a1))
    rhs = ap.systolic_array(5, 3, a0, ap.access(ap.transpose(a1, (1, 0)), 0))
    same(lhs, rhs)
    np.testing.assert_array_equal(rhs.materialize(), ints(1, 7, 5) @ ints(2, 3, 5).T)


def test_im2col_rule1_flatten_then_reshape_is_identity():
    a = ap.access(ap.tensor(ints(3, 2, 3, 4, 5)), 2)
    same(a, ap.reshape(ap.flatten(a), a.access_shape, a.compute_shape))


def test_im2col_rule2_reshape_commutes_with_cartprod():
    a0 = ap.access(ap.tensor(ints(4, 6, 12)), 1)
    a1 = ap.access(ap.tensor(ints(5, 4, 12)), 1)
    s0, s1 = ((2, 3), (3, 4)), ((4,), (3, 4))
    lhs = ap.cart_prod(ap.reshape(a0, *s0), ap.reshape(a1, *s1))
    # ?newShape: access dims concatenated, compute dims (2,) ++ shape0's compute dims
    rhs = ap.reshape(ap.cart_prod(a0, a1), s0[0] + s1[0], (2,) + s0[1])
    same(lhs, rhs)


def test_im2col_rule3_reshape_commutes_with_dotprod():
    a = ap.cart_prod(ap.access(ap.tensor(ints(6, 6, 12)), 1), ap.access(ap.tensor(ints(7, 4, 12)), 1))
    shape = ((2, 3, 4), (2, 3, 4))
    lhs = ap.compute(ap.dotProd, ap.reshape(a, *shape))
    rhs = ap.reshape(ap.compute(ap.dotProd, a), shape[0], ())
    same(lhs, rhs)


@pytest.mark.parametrize("stride,pad", [((1, 1), (0, 0)), ((2, 2), (1, 1)), ((1, 2), (0, 1))])
def test_direct_conv_equals_im2col_conv(stride, pad):
    A, W = ints(8, 2, 3, 8, 7), ints(9, 4, 3, 3, 3)
    same(pg.conv2d(ap.tensor(A), ap.tensor(W), stride, pad),
         pg.conv2d_im2col(ap.tensor(A), ap.tensor(W), stride, pad))


def test_blocking_rule1_slice_concat_identity():
    a = ap.access(ap.tensor(ints(10, 6, 8)), 1)
    for dim, cut in [(0, 2), (1, 5)]:
        same(a, ap.concat(ap.slice_(a, dim, 0, cut), ap.slice_(a, dim, cut, a.shape[dim]), dim))


def test_blocking_rule2_cartprod_concat_on_access_dim():
    a = ap.access(ap.tensor(ints(11, 3, 5)), 1)
    b0, b1 = ap.access(ap.tensor(ints(12, 2, 5)), 1), ap.access(ap.tensor(ints(13, 4, 5)), 1)
    lhs = ap.cart_prod(a, ap.concat(b0, b1, 0))
    rhs = ap.concat(ap.cart_prod(a, b0), ap.cart_prod(a, b1), 0 + a.n_access)   # ?newDim = dim + |a.S_A|
    same(lhs, rhs)


def test_blocking_rule3_cartprod_concat_on_shared_compute_dim():
    a0, a1 = ap.access(ap.tensor(ints(14, 3, 2)), 1), ap.access(ap.tensor(ints(15, 3, 4)), 1)
    a2, a3 = ap.access(ap.tensor(ints(16, 5, 2)), 1), ap.access(ap.tensor(ints(17, 5, 4)), 1)
    lhs = ap.cart_prod(ap.concat(a0, a1, 1), ap.concat(a2, a3, 1))
    # compute dim j = 0 of both sides lands after both access dims and the tuple dim
    rhs = ap.concat(ap.cart_prod(a0, a2), ap.cart_prod(a1, a3), 1 + 1 + 1 + 0)
    same(lhs, rhs)


def test_blocking_rule4_dotprod_concat_on_access_dim():
    a0 = ap.cart_prod(ap.access(ap.tensor(ints(18, 3, 6)), 1), ap.access(ap.tensor(ints(19, 2, 6)), 1))
    a1 = ap.cart_prod(ap.access(ap.tensor(ints(20, 3, 6)), 1), ap.access(ap.tensor(ints(21, 5, 6)), 1))
    same(ap.compute(ap.dotProd, ap.concat(a0, a1, 1)),
         ap.concat(ap.compute(ap.dotProd, a0), ap.compute(ap.dotProd, a1), 1))


def test_blocking_rule5_dotprod_concat_on_compute_dim_is_pairwise_sum():
    x, y = ints(22, 3, 7), ints(23, 4, 7)
    a0 = ap.cart_prod(ap.access(ap.tensor(x[:, :3]), 1), ap.access(ap.tensor(y[:, :3]), 1))
    a1 = ap.cart_prod(ap.access(ap.tensor(x[:, 3:]), 1), ap.access(ap.tensor(y[:, 3:]), 1))
    lhs = ap.compute(ap.dotProd, ap.concat(a0, a1, 3))
    rhs = ap.compute(ap.reduceSum, ap.pair(ap.compute(ap.dotProd, a0), ap.compute(ap.dotProd, a1)))
    same(lhs, rhs)
    np.testing.assert_array_equal(lhs.materialize(), x @ y.T)


@pytest.mark.parametrize("size,block,count", [(32, 16, 8), (32, 8, 64), (16, 16, 1)])
def test_blocked_matmul_equals_plain(size, block, count):
    P, Q = ints(24, size, size), ints(25, size, size)
    prog, n = pg.blocked_matmul(ap.tensor(P), ap.tensor(Q), block)
    assert n == count
    same(prog, pg.matmul(ap.tensor(P), ap.tensor(Q)))
    np.testing.assert_array_equal(prog.materialize(), P @ Q)
