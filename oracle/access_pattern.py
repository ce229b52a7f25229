"""CPU interpreter of Glenside access-pattern programs.

TEST INFRASTRUCTURE ONLY.  This module is the reference the HIP library is
checked against.  Nothing in the product package may import it; only the test
suite, the smoke check and the benchmark's CPU-baseline leg do.  It shares no
code with the HIP path.

What it implements (paper: "Pure Tensor Program Rewriting via Access
Patterns"):

* the access-pattern data model of Sec. 4.1: a tensor of shape S_A ++ S_C seen
  as an S_A-shaped tensor of S_C-shaped elements;
* every transformer of Table 1 (access, transpose, cartProd, windows, slice,
  squeeze, flatten, reshape, pair) plus `concat`, which the blocking rewrites
  of Sec. 5.4 use without a table row;
* the operators of Table 2 (reduceSum, reduceMax, dotProd) under `compute`
  (Sec. 4.3);
* the `systolicArray` construct of the systolic-array rewrite (Sec. 5.2);
* three extensions the paper does not have and the CNN workloads need:
  `pad`, and the scalar operators `relu` and `scale` (documented as
  extensions; pinned only by their textbook definitions).

How it evaluates.  Every node is (shape, n_access, element rule).  The element
rule is written as a *gather*: given one integer array per dimension
(mutually broadcastable) holding positions in the node's own index space,
return the values there.  A
transformer's gather only re-indexes and forwards to its child, so nothing is
materialised until a `compute` node (or the caller) asks for values.  That
makes the same code usable for tiny tensors (evaluate everything) and for
full-size workloads (evaluate a sample of output positions one by one), which
matters because cartProd of a ResNet-sized convolution has billions of
elements.

Arithmetic.  Leaves hold float64 or int64.  Sums and products are taken in
that type, i.e. exactly for integers and in fp64 for floats, with no blocking
or reordering beyond numpy's own reduction over the compute dimensions.
Rounding to the storage type of a GPU buffer (fp32, bf16, int32) is a separate,
explicit step in `oracle.numerics`.

Readings of points the paper leaves open are stated at each node.
"""

from __future__ import annotations

import math
from typing import Callable, Sequence, Tuple

import numpy as np

# Upper bound on the number of leaf reads gathered at once by `compute`.
_CHUNK_ELEMS = 1 << 22

Index = Tuple[np.ndarray, ...]      # one int64 array per dimension, broadcastable


def _prod(xs: Sequence[int]) -> int:
    return int(math.prod(int(x) for x in xs))


def _grid(shape: Sequence[int], lead: int) -> Index:
    """Open index grid over `shape`: array d has extent shape[d] on axis lead+d, 1 elsewhere."""
    n = len(shape)
    out = []
    for d, s in enumerate(shape):
        view = [1] * (lead + n)
        view[lead + d] = int(s)
        out.append(np.arange(int(s), dtype=np.int64).reshape(view))
    return tuple(out)


class AP:
    """An access pattern: shape (S_A, S_C) and a gather rule (Sec. 4.1)."""

    def __init__(self, shape: Sequence[int], n_access: int,
                 gather: Callable[[Index], np.ndarray], kind: str):
        self.shape: Tuple[int, ...] = tuple(int(s) for s in shape)
        self.n_access = int(n_access)
        if not (0 <= self.n_access <= len(self.shape)):
            raise ValueError("access split outside the tensor rank")
        if any(s < 0 for s in self.shape):
            raise ValueError("negative dimension")
        self._gather = gather
        self.kind = kind

    # -- shape views -------------------------------------------------------
    @property
    def rank(self) -> int:
        return len(self.shape)

    @property
    def access_shape(self) -> Tuple[int, ...]:
        return self.shape[: self.n_access]

    @property
    def compute_shape(self) -> Tuple[int, ...]:
        return self.shape[self.n_access:]

    @property
    def ap_shape(self) -> Tuple[Tuple[int, ...], Tuple[int, ...]]:
        """The pair (S_A, S_C) as the paper prints it."""
        return (self.access_shape, self.compute_shape)

    # -- evaluation --------------------------------------------------------
    def gather(self, idx: Sequence[np.ndarray]) -> np.ndarray:
        """Values at the positions idx[0], idx[1], ... (one array per dimension)."""
        idx = tuple(np.asarray(i, dtype=np.int64) for i in idx)
        if len(idx) != self.rank:
            raise ValueError("index rank mismatch")
        for i, s in zip(idx, self.shape):
            if i.size and (i.min() < 0 or i.max() >= s):
                raise IndexError("position outside the access pattern")
        out = self._gather(idx)
        return np.broadcast_to(out, np.broadcast_shapes(*[i.shape for i in idx]) if idx else ())

    def gather_points(self, points: np.ndarray) -> np.ndarray:
        """Values at the rows of an int array points[P, rank]."""
        points = np.asarray(points, dtype=np.int64).reshape(-1, self.rank)
        if self.rank == 0:
            return np.broadcast_to(self._gather(()), (points.shape[0],)).copy()
        return np.array(self.gather(tuple(points[:, d] for d in range(self.rank))))

    def at(self, *index: int):
        """One element."""
        return self.gather_points(np.asarray(index, dtype=np.int64).reshape(1, self.rank))[0]

    def materialize(self) -> np.ndarray:
        """The whole tensor, row-major, shape S_A ++ S_C."""
        if _prod(self.shape) == 0:
            return np.zeros(self.shape, dtype=np.float64)
        if self.rank == 0:
            return np.array(self._gather(()))
        return np.array(np.broadcast_to(self._gather(_grid(self.shape, 0)), self.shape))


# ---------------------------------------------------------------------------
# leaves and `access`
# ---------------------------------------------------------------------------

def tensor(data: np.ndarray) -> AP:
    """A plain tensor (all dimensions compute dimensions until accessed)."""
    data = np.asarray(data)
    if np.issubdtype(data.dtype, np.integer):
        held = data.astype(np.int64)
    else:
        held = data.astype(np.float64)

    def g(idx):
        return held[idx] if held.ndim else held

    return AP(held.shape, 0, g, "tensor")


def access(a: AP, i: int) -> AP:
    """Table 1 `access`: re-split the dimensions at index i; data unchanged."""
    if not (0 <= i <= a.rank):
        raise ValueError("access index outside the rank")
    return AP(a.shape, i, a._gather, "access")


# ---------------------------------------------------------------------------
# Table 1 transformers
# ---------------------------------------------------------------------------

def transpose(a: AP, perm: Sequence[int]) -> AP:
    """Table 1 `transpose`: output dimension t is input dimension perm[t].

    Reading: perm permutes all dimensions of S_A ++ S_C (the table's
    "(0..n-1)" for dims a_0..a_n is an off-by-one; the listings use
    (1 0) on rank 2 and (0 3 1 2) on rank 4) and the access split stays where
    it was: ((N),(O)) -> ((O),(N)) in Sec. 4.2.
    """
    perm = tuple(int(p) for p in perm)
    if sorted(perm) != list(range(a.rank)):
        raise ValueError("not a permutation of the dimensions")
    shape = tuple(a.shape[p] for p in perm)

    def g(idx):
        src = [None] * len(perm)
        for t, p in enumerate(perm):
            src[p] = idx[t]
        return a._gather(tuple(src))

    return AP(shape, a.n_access, g, "transpose")


def cart_prod(a: AP, b: AP) -> AP:
    """Table 1 `cartProd`: ((a..),(c..)) x ((b..),(c..)) -> ((a..,b..),(2,c..)).

    Element rule (Sec. 4.2: a 2-tuple of the inputs' compute dimensions, first
    input first): out[a.., b.., 0, c..] = A[a.., c..], out[a.., b.., 1, c..] =
    B[b.., c..].
    """
    if a.compute_shape != b.compute_shape:
        raise ValueError("cartProd needs equal compute dimensions")
    na, nb = a.n_access, b.n_access
    shape = a.access_shape + b.access_shape + (2,) + a.compute_shape

    def g(idx):
        sel = idx[na + nb]
        c = idx[na + nb + 1:]
        va = a._gather(idx[:na] + c)
        vb = b._gather(idx[na:na + nb] + c)
        return np.where(sel == 0, va, vb)

    return AP(shape, na + nb, g, "cartProd")


def windows_out_dim(b: int, w: int, s: int) -> int:
    """Table 1 `windows`: b' = ceil((b - (w - 1)) / s)  (the table's k_i is w_i)."""
    return -((-(b - (w - 1))) // s)


def windows(a: AP, window: Sequence[int], stride: Sequence[int]) -> AP:
    """Table 1 `windows`: ((a..),(b..)) -> ((a.., b'..),(w..)).

    Element rule (the table gives only the shape; the conv2d and max-pool
    equations of Sec. 5.1 force it): out[a.., p.., q..] = A[a.., p_i*s_i + q_i ..].
    Windows that would run past the end do not exist.
    """
    window = tuple(int(w) for w in window)
    stride = tuple(int(s) for s in stride)
    nc = len(a.compute_shape)
    if len(window) != nc or len(stride) != nc:
        raise ValueError("window/stride rank must equal the compute rank")
    for b, w, s in zip(a.compute_shape, window, stride):
        if w < 1 or s < 1 or w > b:
            raise ValueError("window must fit inside the compute dimensions")
    outer = tuple(windows_out_dim(b, w, s) for b, w, s in zip(a.compute_shape, window, stride))
    na = a.n_access
    shape = a.access_shape + outer + window

    def g(idx):
        p = idx[na:na + nc]
        q = idx[na + nc:]
        inner = tuple(p[i] * stride[i] + q[i] for i in range(nc))
        return a._gather(idx[:na] + inner)

    return AP(shape, na + nc, g, "windows")


def slice_(a: AP, dim: int, lo: int, hi: int) -> AP:
    """Table 1 `slice`: keep [lo, hi) of dimension dim (argument order as in Fig. 7)."""
    if not (0 <= dim < a.rank) or not (0 <= lo <= hi <= a.shape[dim]):
        raise ValueError("bad slice")
    shape = a.shape[:dim] + (hi - lo,) + a.shape[dim + 1:]

    def g(idx):
        return a._gather(idx[:dim] + (idx[dim] + lo,) + idx[dim + 1:])

    return AP(shape, a.n_access, g, "slice")


def squeeze(a: AP, dim: int) -> AP:
    """Table 1 `squeeze`: drop a size-1 dimension.

    Reading: the access split moves left when the dropped dimension was an
    access dimension, as Fig. 2a needs: ((N,1,H',W',O),()) -> ((N,H',W',O),()).
    """
    if not (0 <= dim < a.rank) or a.shape[dim] != 1:
        raise ValueError("squeeze needs a size-1 dimension")
    shape = a.shape[:dim] + a.shape[dim + 1:]
    n_access = a.n_access - 1 if dim < a.n_access else a.n_access

    def g(idx):
        return a._gather(idx[:dim] + (np.zeros((), dtype=np.int64),) + idx[dim:])

    return AP(shape, n_access, g, "squeeze")


def _ravel(multi: Index, shape: Sequence[int]) -> np.ndarray:
    """Multi-index -> row-major flat position."""
    flat = np.zeros((), dtype=np.int64)
    for d in range(len(shape)):
        flat = flat * shape[d] + multi[d]
    return flat


def _unravel(flat: np.ndarray, shape: Sequence[int]) -> Index:
    """Row-major flat position -> multi-index."""
    out = [None] * len(shape)
    rem = flat
    for d in range(len(shape) - 1, -1, -1):
        out[d] = rem % shape[d]
        rem = rem // shape[d]
    return tuple(out)


def reshape(a: AP, access_shape: Sequence[int], compute_shape: Sequence[int]) -> AP:
    """Table 1 `reshape`: to the literal shape ((c..),(d..)), each side keeping its product.

    Row-major order on each side is kept, so dense data is unchanged.
    """
    access_shape = tuple(int(x) for x in access_shape)
    compute_shape = tuple(int(x) for x in compute_shape)
    if _prod(access_shape) != _prod(a.access_shape) or _prod(compute_shape) != _prod(a.compute_shape):
        raise ValueError("reshape must keep the product of each side")
    na_new, old_a, old_c = len(access_shape), a.access_shape, a.compute_shape

    def g(idx):
        fa = _ravel(idx[:na_new], access_shape)
        fc = _ravel(idx[na_new:], compute_shape)
        return a._gather(_unravel(fa, old_a) + _unravel(fc, old_c))

    return AP(access_shape + compute_shape, na_new, g, "reshape")


def flatten(a: AP) -> AP:
    """Table 1 `flatten`: ((a..),(b..)) -> ((prod a),(prod b)); an empty side stays empty."""
    acc = (_prod(a.access_shape),) if a.access_shape else ()
    cmp_ = (_prod(a.compute_shape),) if a.compute_shape else ()
    out = reshape(a, acc, cmp_)
    out.kind = "flatten"
    return out


def pair(a: AP, b: AP) -> AP:
    """Table 1 `pair`: two patterns of one shape -> ((a..),(2, c..)); the 2 leads the compute dims."""
    if a.ap_shape != b.ap_shape:
        raise ValueError("pair needs two access patterns of the same shape")
    na = a.n_access
    shape = a.access_shape + (2,) + a.compute_shape

    def g(idx):
        src = idx[:na] + idx[na + 1:]
        return np.where(idx[na] == 0, a._gather(src), b._gather(src))

    return AP(shape, na, g, "pair")


def concat(a: AP, b: AP, dim: int) -> AP:
    """`concat` of the blocking rewrites (Sec. 5.4): join along dim; other dims and split equal."""
    if a.rank != b.rank or a.n_access != b.n_access or not (0 <= dim < a.rank):
        raise ValueError("concat needs patterns of equal rank and access split")
    for d in range(a.rank):
        if d != dim and a.shape[d] != b.shape[d]:
            raise ValueError("concat: dimensions other than dim must agree")
    cut = a.shape[dim]
    shape = a.shape[:dim] + (cut + b.shape[dim],) + a.shape[dim + 1:]

    def g(idx):
        in_b = idx[dim] >= cut
        if cut == 0:
            return b._gather(idx)
        if b.shape[dim] == 0:
            return a._gather(idx)
        ia = idx[:dim] + (np.where(in_b, 0, idx[dim]),) + idx[dim + 1:]
        ib = idx[:dim] + (np.where(in_b, idx[dim] - cut, 0),) + idx[dim + 1:]
        return np.where(in_b, b._gather(ib), a._gather(ia))

    return AP(shape, a.n_access, g, "concat")


def pad(a: AP, dim: int, lo: int, hi: int, value) -> AP:
    """EXTENSION (not in the paper): grow dimension dim by lo cells before and hi after, filled with value."""
    if not (0 <= dim < a.rank) or lo < 0 or hi < 0:
        raise ValueError("bad pad")
    size = a.shape[dim]
    shape = a.shape[:dim] + (size + lo + hi,) + a.shape[dim + 1:]

    def g(idx):
        pos = idx[dim] - lo
        inside = (pos >= 0) & (pos < size)
        vals = a._gather(idx[:dim] + (np.where(inside, pos, 0),) + idx[dim + 1:])
        return np.where(inside, vals, np.asarray(value, dtype=vals.dtype))

    return AP(shape, a.n_access, g, "pad")


# ---------------------------------------------------------------------------
# Table 2 operators and `compute`
# ---------------------------------------------------------------------------

class Operator:
    """An operator: maps an S_C-shaped element to a result element (Table 2)."""

    def __init__(self, name: str, out_shape: Callable[[Tuple[int, ...]], Tuple[int, ...]],
                 apply: Callable[[np.ndarray, int], np.ndarray]):
        self.name = name
        self.out_shape = out_shape
        self.apply = apply  # (values[..., *S_C], number of compute dims) -> values[..., *out]


def _reduce_axes(n: int) -> Tuple[int, ...]:
    return tuple(range(-n, 0))


def _reduce_sum(v, n):
    return v.sum(axis=_reduce_axes(n)) if n else v


def _reduce_max(v, n):
    if n and _prod(v.shape[-n:]) == 0:
        raise ValueError("reduceMax of an empty element")
    return v.max(axis=_reduce_axes(n)) if n else v


def _dot_prod(v, n):
    # (t, s_0..s_n) -> (): multiply along the leading (tuple) axis, then sum everything.
    if n < 1 or v.shape[-n] < 2:
        raise ValueError("dotProd needs a leading tuple dimension of at least 2")
    prod = np.prod(v, axis=-n)
    return prod.sum(axis=_reduce_axes(n - 1)) if n > 1 else prod


reduceSum = Operator("reduceSum", lambda sc: (), _reduce_sum)
reduceMax = Operator("reduceMax", lambda sc: (), _reduce_max)
dotProd = Operator("dotProd", lambda sc: (), _dot_prod)


def _scalar_only(sc):
    if sc != ():
        raise ValueError("scalar operator needs an empty compute shape")
    return ()


#: EXTENSION (not in the paper): max(x, 0) on scalar elements.
relu = Operator("relu", _scalar_only, lambda v, n: np.maximum(v, np.zeros((), dtype=v.dtype)))


def scale(alpha: float) -> Operator:
    """EXTENSION (not in the paper): multiply scalar elements by alpha (in fp64)."""
    return Operator("scale", _scalar_only, lambda v, n: v.astype(np.float64) * np.float64(alpha))


def compute(op: Operator, a: AP) -> AP:
    """Sec. 4.3 `compute`: apply op to the element at every access index; S_A is unchanged."""
    na = a.n_access
    sc = a.compute_shape
    if tuple(op.out_shape(sc)) != ():
        raise NotImplementedError("all operators here return scalars")
    nsc = len(sc)
    pc = max(_prod(sc), 1)

    def g(idx):
        lead_shape = np.broadcast_shapes(*[i.shape for i in idx]) if idx else ()
        flat = [np.broadcast_to(i, lead_shape).reshape(-1) for i in idx]
        n = _prod(lead_shape)
        cgrid = _grid(sc, 1)                      # arrays of shape [1, *S_C-open]
        step = max(1, _CHUNK_ELEMS // pc)
        parts = []
        for lo in range(0, n, step):
            blk = tuple(f[lo:lo + step].reshape((-1,) + (1,) * nsc) for f in flat)
            m = min(step, n - lo)
            vals = np.broadcast_to(a._gather(blk + cgrid), (m,) + sc)
            parts.append(np.asarray(op.apply(vals, nsc)).reshape(m))
        if not parts:
            return np.zeros(lead_shape, dtype=np.float64)
        return np.concatenate(parts).reshape(lead_shape)

    return AP(a.access_shape, na, g, "compute:" + op.name)


def systolic_array(rows: int, cols: int, a0: AP, w: AP) -> AP:
    """The `systolicArray` construct of the systolic-array rewrite (Sec. 5.2).

    a0 : ((batch),(rows)); w : ((),(rows, cols)), i.e. the weights read all at
    once and laid out transposed.  Result ((batch, cols),()) with
    out[b, c] = sum_r a0[b, r] * w[r, c]  (the result shape is fixed by the
    rewrite asserting equality with `compute dotProd (cartProd a0 a1)`).
    """
    if a0.n_access != 1 or a0.rank != 2 or a0.shape[1] != rows:
        raise ValueError("systolicArray: a0 must be ((batch),(rows))")
    if w.n_access != 0 or w.shape != (rows, cols):
        raise ValueError("systolicArray: w must be ((),(rows, cols))")
    batch = a0.shape[0]
    r = np.arange(rows, dtype=np.int64)

    def g(idx):
        b = idx[0][..., None]
        c = idx[1][..., None]
        return (a0._gather((b, r)) * w._gather((r, c))).sum(axis=-1)

    return AP((batch, cols), 2, g, "systolicArray")
