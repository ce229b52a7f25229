"""Programs as text, without a GPU: the oracle's text interpreter against the pinned builders and
brute-force loops, and the library's host-side shape rules and rewrites (Figs. 3, 4, 6) checked
through the oracle: a rewritten program must denote the same tensor as the original."""

import numpy as np
import pytest
import torch

from oracle import access_pattern as ap, brute, programs as pg, sexpr
from paper_2105_09377_amd import binding as gs
import listings


def rng(seed):
    return np.random.default_rng(seed)


CONV_INTS = dict(C=3, Kh=3, Kw=2, Sh=2, Sw=1)


def conv_inputs():
    r = rng(41)
    return r.integers(-8, 9, (2, 3, 9, 8)), r.integers(-8, 9, (5, 3, 3, 2))


# -- the oracle's reader / interpreter of program text ------------------------------------------

def test_parse_round_trip_and_errors():
    tree = sexpr.parse("(compute dotProd (cartProd (access a 1) (access b 1)))")
    assert tree == ["compute", "dotProd", ["cartProd", ["access", "a", 1], ["access", "b", 1]]]
    assert sexpr.parse(sexpr.to_text(tree)) == tree
    for bad in ["(access a 1", "access a 1)", "(a) (b)", ""]:
        with pytest.raises(ValueError):
            sexpr.parse(bad)


def test_text_conv2d_is_the_listing_and_the_loops():
    A, W = conv_inputs()
    got = sexpr.evaluate(listings.CONV2D, {"activations": A, "weights": W}, CONV_INTS)
    assert got.ap_shape == ((2, 5, 4, 7), ())
    want = brute.conv2d(A, W, (2, 1))
    np.testing.assert_array_equal(got.materialize(), want)
    np.testing.assert_array_equal(got.materialize(), pg.conv2d(ap.tensor(A), ap.tensor(W), (2, 1)).materialize())


def test_text_matmul_maxpool_pad_pair_concat():
    r = rng(43)
    P, Q = r.integers(-9, 9, (6, 7)), r.integers(-9, 9, (7, 4))
    got = sexpr.evaluate(listings.MATMUL, {"activations": P, "weights": Q})
    np.testing.assert_array_equal(got.materialize(), P @ Q)
    X = r.integers(-50, 50, (2, 3, 7, 8))
    mp = sexpr.evaluate(listings.MAXPOOL, {"activations": X}, dict(Kh=3, Kw=2, Sh=2, Sw=2))
    np.testing.assert_array_equal(mp.materialize(), brute.max_pool2d(X, (3, 2), (2, 2)))
    A, W = conv_inputs()
    ints = dict(CONV_INTS, Ph=1, Pw=2)
    padded = sexpr.evaluate(listings.CONV2D_PADDED, {"activations": A, "weights": W}, ints)
    np.testing.assert_array_equal(padded.materialize(), brute.conv2d(A, W, (2, 1), (1, 2)))
    s = sexpr.evaluate("(compute reduceSum (pair (access a 2) (access b 2)))", {"a": P, "b": P + 1})
    np.testing.assert_array_equal(s.materialize(), 2 * P + 1)
    c = sexpr.evaluate("(concat (slice (access a 1) 1 0 3) (slice (access a 1) 1 3 7) 1)", {"a": P})
    np.testing.assert_array_equal(c.materialize(), P)


# -- the library's shape rules ------------------------------------------------------------------

def meta(**arrays):
    return {k: (tuple(v.shape), torch.int8) for k, v in arrays.items()}


def test_program_shape_follows_the_oracle():
    A, W = conv_inputs()
    for text, tensors, ints in [
        (listings.CONV2D, dict(activations=A, weights=W), CONV_INTS),
        (listings.CONV2D_PADDED, dict(activations=A, weights=W), dict(CONV_INTS, Ph=1, Pw=2)),
        (listings.MATMUL, dict(activations=A[0, 0], weights=A[0, 1].T.copy()), {}),
        (listings.MAXPOOL, dict(activations=A), dict(Kh=3, Kw=2, Sh=2, Sw=2)),
        ("(flatten (windows (access activations 1) (shape 3 3 3) (shape 1 1 1)))", dict(activations=A), {}),
        ("(pair (access activations 2) (access activations 2))", dict(activations=A), {}),
    ]:
        want = sexpr.evaluate(text, tensors, ints)
        shape, na, _ = gs.program_shape(text, meta(**tensors), ints)
        assert (shape[:na], shape[na:]) == want.ap_shape, text


def test_program_shape_errors():
    A, W = conv_inputs()
    m = meta(activations=A, weights=W)
    def status(text, ints=None):
        with pytest.raises(gs.GlensideError) as e:
            gs.program_shape(text, m, ints or {})
        return e.value.status
    assert status("(access activations 1") == gs.GS_ERR_UNSUPPORTED          # unbalanced
    assert status("(access nothing 1)") == gs.GS_ERR_NULL                    # unknown tensor
    assert status("(access activations 9)") == gs.GS_ERR_RANK
    assert status("(frobnicate activations)") == gs.GS_ERR_UNSUPPORTED
    assert status("(windows (access activations 1) (shape 3 3) (shape 1 1))") == gs.GS_ERR_RANK
    assert status("(windows (access activations 1) (shape 3 99 3) (shape 1 1 1))") == gs.GS_ERR_SHAPE
    assert status("(cartProd (access activations 1) (access weights 2))") == gs.GS_ERR_SHAPE
    assert status("(squeeze (access activations 1) 0)") == gs.GS_ERR_SHAPE
    assert status("(reshape (access activations 1) (shape 4) (shape 3 9 8))") == gs.GS_ERR_SHAPE
    assert status("(slice (access activations 1) 0 1 5)") == gs.GS_ERR_SHAPE
    assert status("(compute dotProd (access activations 1))") == gs.GS_ERR_SHAPE   # no tuple dimension
    assert status(listings.CONV2D) == gs.GS_ERR_UNSUPPORTED                  # C, Kh ... not bound


# -- the rewrites --------------------------------------------------------------------------------

def test_im2col_rewrite_derives_the_flattened_program():
    A, W = conv_inputs()
    m = meta(activations=A, weights=W)
    text = gs.program_rewrite(listings.CONV2D, "im2col", m, CONV_INTS)
    tree = sexpr.parse(text)
    # the shape of Fig. 5: transpose (squeeze (reshape (compute dotProd (cartProd (flatten (windows
    # ...)) (flatten (access weights 1)))) ?shape) 1) (list 0 3 1 2)
    assert tree[0] == "transpose" and tree[2] == ["list", 0, 3, 1, 2]
    sq = tree[1]
    assert sq[0] == "squeeze" and sq[2] == 1
    rs = sq[1]
    assert rs[0] == "reshape" and rs[2] == ["shape", 2, 1, 4, 7, 5] and rs[3] == ["shape"]
    dp = rs[1]
    assert dp[:2] == ["compute", "dotProd"] and dp[2][0] == "cartProd"
    left, right = dp[2][1], dp[2][2]
    assert left[0] == "flatten" and left[1][0] == "windows"
    assert right == ["flatten", ["access", "weights", 1]]
    # equality: both programs denote the same tensor (bit for bit on integers)
    tensors = {"activations": A, "weights": W}
    np.testing.assert_array_equal(sexpr.evaluate(text, tensors, CONV_INTS).materialize(),
                                  sexpr.evaluate(listings.CONV2D, tensors, CONV_INTS).materialize())
    # the flattened operand is the im2col matrix
    cols = sexpr.evaluate(sexpr.to_text(left), tensors, CONV_INTS)
    assert cols.ap_shape == ((2 * 4 * 7,), (3 * 3 * 2,))


@pytest.mark.parametrize("dims,blocks,products", [((32, 32, 32), (16, 16, 16), 8), ((48, 32, 40), (16, 32, 8), 15),
                                                  ((20, 24, 36), (16, 16, 16), 2 * 2 * 3)])
def test_blocking_rewrite_derives_block_products(dims, blocks, products):
    m_, n_, k_ = dims
    r = rng(47)
    P, Q = r.integers(-9, 9, (m_, k_)), r.integers(-9, 9, (k_, n_))
    tensors = {"activations": P, "weights": Q}
    text = gs.program_rewrite(listings.MATMUL, "block", meta(**tensors), params=blocks)
    assert text.count("(cartProd") == products          # the 32x32 case: the paper's eight 16x16 products
    assert text.count("(compute dotProd (cartProd") == products
    got = sexpr.evaluate(text, tensors)
    assert got.ap_shape == ((m_, n_), ())
    np.testing.assert_array_equal(got.materialize(), P @ Q)
    # every product is of blocks: no cartProd operand is larger than a block
    def operands(tree, out):
        if isinstance(tree, list):
            if tree and tree[0] == "cartProd":
                out.append((tree[1], tree[2]))
            for t in tree:
                operands(t, out)
        return out
    for a, b in operands(sexpr.parse(text), []):
        sa = sexpr.evaluate(sexpr.to_text(a), tensors).shape
        sb = sexpr.evaluate(sexpr.to_text(b), tensors).shape
        assert sa[0] <= blocks[0] and sb[0] <= blocks[1] and sa[1] <= blocks[2] and sa[1] == sb[1]


def test_systolic_rewrite():
    r = rng(53)
    P, Q = r.integers(-9, 9, (5, 7)), r.integers(-9, 9, (4, 7))
    tensors = {"a0": P, "a1": Q}
    lhs = "(compute dotProd (cartProd (access a0 1) (access a1 1)))"
    text = gs.program_rewrite(lhs, "systolic", meta(**tensors))
    assert sexpr.parse(text) == ["systolicArray", 7, 4, ["access", "a0", 1],
                                 ["access", ["transpose", ["access", "a1", 1], ["list", 1, 0]], 0]]
    np.testing.assert_array_equal(sexpr.evaluate(text, tensors).materialize(), P @ Q.T)


def test_rewrite_refuses_programs_without_the_pattern():
    A, _ = conv_inputs()
    with pytest.raises(gs.GlensideError) as e:
        gs.program_rewrite(listings.MAXPOOL, "im2col", meta(activations=A), dict(Kh=2, Kw=2, Sh=2, Sw=2))
    assert e.value.status == gs.GS_ERR_UNSUPPORTED
    with pytest.raises(gs.GlensideError):
        gs.program_rewrite(listings.MATMUL, "unknown-strategy", meta(activations=A[0, 0], weights=A[0, 0].T.copy()))


def test_rewrites_on_random_shapes():
    """Seeded sweep: random matrix sizes and block sizes (ragged last blocks, blocks larger than the
    matrix, blocks of one), random convolution shapes and strides -- the rewritten program always
    denotes the tensor the original does."""
    r = rng(59)
    for _ in range(25):
        m_, n_, k_ = (int(v) for v in r.integers(1, 40, 3))
        blocks = tuple(int(v) for v in r.integers(1, 48, 3))
        P, Q = r.integers(-9, 9, (m_, k_)), r.integers(-9, 9, (k_, n_))
        tensors = {"activations": P, "weights": Q}
        if -(-m_ // blocks[0]) * -(-n_ // blocks[1]) * -(-k_ // blocks[2]) > 400:
            continue
        text = gs.program_rewrite(listings.MATMUL, "block", meta(**tensors), params=blocks)
        np.testing.assert_array_equal(sexpr.evaluate(text, tensors).materialize(), P @ Q, err_msg=str((m_, n_, k_, blocks)))
        sys_text = gs.program_rewrite("(compute dotProd (cartProd (access activations 1) (access (transpose (access weights 1) (list 1 0)) 1)))",
                                      "systolic", meta(**tensors))
        np.testing.assert_array_equal(sexpr.evaluate(sys_text, tensors).materialize(), P @ Q)
    for _ in range(12):
        n, c, o = (int(v) for v in r.integers(1, 4, 3))
        kh, kw, sh, sw = (int(v) for v in r.integers(1, 4, 4))
        h, w = int(r.integers(kh, kh + 7)), int(r.integers(kw, kw + 7))
        A, W = r.integers(-8, 9, (n, c, h, w)), r.integers(-8, 9, (o, c, kh, kw))
        ints = dict(C=c, Kh=kh, Kw=kw, Sh=sh, Sw=sw)
        tensors = {"activations": A, "weights": W}
        text = gs.program_rewrite(listings.CONV2D, "im2col", meta(**tensors), ints)
        want = brute.conv2d(A, W, (sh, sw), (0, 0))
        np.testing.assert_array_equal(sexpr.evaluate(text, tensors, ints).materialize(), want, err_msg=str(ints))
        np.testing.assert_array_equal(sexpr.evaluate(listings.CONV2D, tensors, ints).materialize(), want)
