"""The paper's kernel specifications, written as access-pattern programs.

TEST INFRASTRUCTURE ONLY (see `oracle.access_pattern`).  Each function builds
the expression of one listing of the paper out of the interpreter's nodes and
returns the un-evaluated access pattern; call `.materialize()` for the whole
result or `.gather(idx)` for sampled positions.
"""

from __future__ import annotations

from typing import Optional, Sequence

from . import access_pattern as ap


def _padded_activations(activations: ap.AP, pad_hw: Sequence[int], value) -> ap.AP:
    """EXTENSION: symmetric spatial padding of an (N, C, H, W) tensor.

    The paper has no padding; a padded convolution / pooling is *defined* here
    as the paper's program applied to an explicitly padded tensor.
    """
    ph, pw = int(pad_hw[0]), int(pad_hw[1])
    x = activations
    if ph:
        x = ap.pad(x, 2, ph, ph, value)
    if pw:
        x = ap.pad(x, 3, pw, pw, value)
    return x


def conv2d(activations: ap.AP, weights: ap.AP, stride: Sequence[int],
           pad_hw: Sequence[int] = (0, 0)) -> ap.AP:
    """Fig. 2a: activations (N,C,H,W), weights (O,C,Kh,Kw) -> ((N,O,H',W'),()).

    Follows the listing (windows first in the Cartesian product), which is
    the only order consistent with `squeeze 1` and `transpose (0 3 1 2)`.
    """
    o, c, kh, kw = weights.shape
    x = _padded_activations(activations, pad_hw, 0)
    win = ap.windows(ap.access(x, 1), (c, kh, kw), (1, int(stride[0]), int(stride[1])))
    cp = ap.cart_prod(win, ap.access(weights, 1))
    dp = ap.compute(ap.dotProd, cp)
    return ap.transpose(ap.squeeze(dp, 1), (0, 3, 1, 2))


def depthwise_conv2d(activations: ap.AP, weights: ap.AP, stride: Sequence[int],
                     pad_hw: Sequence[int] = (0, 0)) -> ap.AP:
    """Depth-wise windows, written with Table 1 / Table 2 operators only: activations (N,C,H,W),
    weights (C,1,Kh,Kw) -> ((N,C,H',W'),()).  Channel c of the activations and filter c of the
    weights are cut out with `slice`, put through the program of Fig. 2a (a one-channel,
    one-filter convolution), and the C results are joined with `concat` along dimension 1."""
    c = activations.shape[1]
    assert weights.shape[0] == c and weights.shape[1] == 1
    result = None
    for ch in range(c):
        one = conv2d(ap.slice_(activations, 1, ch, ch + 1), ap.slice_(weights, 0, ch, ch + 1), stride, pad_hw)
        result = one if result is None else ap.concat(result, one, 1)
    return result


def conv2d_im2col(activations: ap.AP, weights: ap.AP, stride: Sequence[int],
                  pad_hw: Sequence[int] = (0, 0)) -> ap.AP:
    """Fig. 5: the im2col form; `?shape` is the shape of the direct form's dotProd result."""
    o, c, kh, kw = weights.shape
    x = _padded_activations(activations, pad_hw, 0)
    win = ap.windows(ap.access(x, 1), (c, kh, kw), (1, int(stride[0]), int(stride[1])))
    n, one, h_out, w_out = win.access_shape
    cols = ap.flatten(win)                               # ((N*1*H'*W'),(C*Kh*Kw))
    filt = ap.flatten(ap.access(weights, 1))             # ((O),(C*Kh*Kw))
    dp = ap.compute(ap.dotProd, ap.cart_prod(cols, filt))   # ((N*1*H'*W', O),())
    rs = ap.reshape(dp, (n, one, h_out, w_out, o), ())
    return ap.transpose(ap.squeeze(rs, 1), (0, 3, 1, 2))


def im2col_matrix(activations: ap.AP, window_chw: Sequence[int], stride: Sequence[int],
                  pad_hw: Sequence[int] = (0, 0)) -> ap.AP:
    """The flattened windows of Fig. 5: ((N*1*H'*W'),(C*Kh*Kw))."""
    c, kh, kw = (int(v) for v in window_chw)
    x = _padded_activations(activations, pad_hw, 0)
    win = ap.windows(ap.access(x, 1), (c, kh, kw), (1, int(stride[0]), int(stride[1])))
    return ap.flatten(win)


def matmul(activations: ap.AP, weights: ap.AP) -> ap.AP:
    """Fig. 2b: activations (M,N), weights (N,O) -> ((M,O),())."""
    return ap.compute(ap.dotProd, ap.cart_prod(
        ap.access(activations, 1), ap.transpose(ap.access(weights, 1), (1, 0))))


def cartesian_dot(a0: ap.AP, a1: ap.AP) -> ap.AP:
    """Left-hand side of the systolic-array rewrite: compute dotProd (cartProd a0 a1)."""
    return ap.compute(ap.dotProd, ap.cart_prod(a0, a1))


def max_pool2d(activations: ap.AP, window: Sequence[int], stride: Sequence[int],
               pad_hw: Sequence[int] = (0, 0), pad_value=None) -> ap.AP:
    """Fig. 2c: activations (N,C,H,W) -> ((N,C,H',W'),()); padding (extension) uses pad_value."""
    x = activations
    if any(int(p) for p in pad_hw):
        if pad_value is None:
            raise ValueError("padded max-pool needs the lowest value of the storage type")
        x = _padded_activations(activations, pad_hw, pad_value)
    win = ap.windows(ap.access(x, 2), (int(window[0]), int(window[1])),
                     (int(stride[0]), int(stride[1])))
    return ap.compute(ap.reduceMax, win)


def add(a: ap.AP, b: ap.AP) -> ap.AP:
    """Element-wise sum in the paper's idiom: compute reduceSum (pair a b) (Sec. 5.4)."""
    return ap.compute(ap.reduceSum, ap.pair(a, b))


def blocked_matmul(activations: ap.AP, weights: ap.AP, block: int) -> tuple:
    """Fig. 7 generalised: a square-blocked matmul built from slice/concat/pair.

    activations (M,K), weights (K,O) in the layout of Fig. 2b, every dimension
    a multiple of `block`.  Returns (program, number of block multiplications).
    K blocks are folded left to right with compute reduceSum (pair ...), O
    blocks and M blocks are joined with concat on access dimensions 1 and 0.
    """
    m, k = activations.shape
    k2, o = weights.shape
    if k != k2 or m % block or k % block or o % block:
        raise ValueError("dimensions must be multiples of the block size")
    a = ap.access(activations, 1)
    w = ap.access(weights, 1)
    count = 0
    rows = None
    for mi in range(0, m, block):
        row = None
        for oi in range(0, o, block):
            acc = None
            for ki in range(0, k, block):
                a_blk = ap.slice_(ap.slice_(a, 0, mi, mi + block), 1, ki, ki + block)
                w_blk = ap.transpose(
                    ap.slice_(ap.slice_(w, 0, ki, ki + block), 1, oi, oi + block), (1, 0))
                part = ap.compute(ap.dotProd, ap.cart_prod(a_blk, w_blk))
                count += 1
                acc = part if acc is None else ap.compute(ap.reduceSum, ap.pair(acc, part))
            row = acc if row is None else ap.concat(row, acc, 1)
        rows = row if rows is None else ap.concat(rows, row, 0)
    return rows, count
