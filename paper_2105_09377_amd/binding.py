"""ctypes binding of `libglenside.so` (declared in include/glenside.h).

Argument marshalling only: every function here builds `gs_ap` descriptors from torch tensors
(device memory and the current stream come from torch), calls the C entry point of the same
name, and raises `GlensideError` on a non-zero status.  No arithmetic happens in Python.  There is no
fallback: if the library has not been built, loading fails with an error.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libglenside.so")

GS_MAX_RANK = 8
GS_I8, GS_I32, GS_BF16, GS_F32, GS_F8 = 0, 1, 2, 3, 4
GS_SUM, GS_MAX = 0, 1
GS_ACT_NONE, GS_ACT_RELU = 0, 1
GS_PAD_ZERO, GS_PAD_LOWEST = 0, 1
(GS_OK, GS_ERR_NULL, GS_ERR_RANK, GS_ERR_SHAPE, GS_ERR_DTYPE, GS_ERR_UNSUPPORTED,
 GS_ERR_WORKSPACE, GS_ERR_LAUNCH) = range(8)

_DTYPES = {torch.int8: GS_I8, torch.int32: GS_I32, torch.bfloat16: GS_BF16, torch.float32: GS_F32,
           torch.float8_e4m3fn: GS_F8}

EXPORTS = (
    "glenside_status_string", "glenside_windows_out_shape", "glenside_access_windows",
    "glenside_cartesian_dot", "glenside_conv2d_direct", "glenside_conv2d_im2col",
    "glenside_conv2d_direct_workspace", "glenside_conv2d_im2col_workspace", "glenside_reduce",
    "glenside_windows_reduce", "glenside_pair_reduce", "glenside_conv2d_pack_weights",
    "glenside_conv2d_direct_packed", "glenside_transpose", "glenside_slice", "glenside_concat",
    "glenside_pad", "glenside_pair", "glenside_cartesian_dot_blocked",
    "glenside_conv2d_direct_static", "glenside_conv2d_direct_static_limit",
    "glenside_program_shape", "glenside_program_eval", "glenside_program_workspace",
    "glenside_program_rewrite", "glenside_depthwise_conv2d",
)


class gs_ap(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("rank", ctypes.c_int32),
                ("n_access", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("shape", ctypes.c_int64 * GS_MAX_RANK)]


class gs_named_ap(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("tensor", gs_ap)]


class gs_named_int(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("value", ctypes.c_int64)]


class GlensideError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library (never builds, never falls back)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2105_09377_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        ap_p, i64_p, vp = ctypes.POINTER(gs_ap), ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p
        L.glenside_status_string.restype = ctypes.c_char_p
        L.glenside_status_string.argtypes = [ctypes.c_int]
        L.glenside_windows_out_shape.argtypes = [ap_p, i64_p, i64_p, i64_p, i64_p, ap_p]
        L.glenside_access_windows.argtypes = [ap_p, i64_p, i64_p, i64_p, i64_p, ctypes.c_int, ap_p, vp]
        L.glenside_cartesian_dot.argtypes = [ap_p, ap_p, ap_p, ctypes.c_int, vp, ctypes.c_size_t, vp]
        conv = [ap_p, ap_p, i64_p, i64_p, ap_p, ctypes.c_int, ap_p, vp, ctypes.c_size_t, vp]
        L.glenside_conv2d_direct.argtypes = conv
        L.glenside_conv2d_im2col.argtypes = conv
        for f in (L.glenside_conv2d_direct_workspace, L.glenside_conv2d_im2col_workspace):
            f.restype = ctypes.c_size_t
            f.argtypes = [ap_p, ap_p, i64_p, i64_p]
        L.glenside_conv2d_direct_static.argtypes = [ap_p, ap_p, i64_p, i64_p, ap_p, ctypes.c_int, ap_p, vp]
        L.glenside_conv2d_direct_static_limit.restype = ctypes.c_size_t
        L.glenside_conv2d_direct_static_limit.argtypes = []
        nap_p, nint_p = ctypes.POINTER(gs_named_ap), ctypes.POINTER(gs_named_int)
        prog = [ctypes.c_char_p, nap_p, ctypes.c_int, nint_p, ctypes.c_int]
        L.glenside_program_shape.argtypes = prog + [ap_p]
        L.glenside_program_workspace.argtypes = prog
        L.glenside_program_workspace.restype = ctypes.c_size_t
        L.glenside_program_eval.argtypes = prog + [ap_p, vp, ctypes.c_size_t, vp]
        L.glenside_program_rewrite.argtypes = [ctypes.c_char_p, ctypes.c_char_p, i64_p, ctypes.c_int, nap_p,
                                               ctypes.c_int, nint_p, ctypes.c_int, ctypes.c_char_p,
                                               ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        L.glenside_conv2d_pack_weights.argtypes = [ap_p, vp, ctypes.c_size_t, vp]
        L.glenside_conv2d_direct_packed.argtypes = conv
        L.glenside_reduce.argtypes = [ap_p, ctypes.c_int, ctypes.c_float, ap_p, vp]
        L.glenside_windows_reduce.argtypes = [ap_p, i64_p, i64_p, i64_p, i64_p, ctypes.c_int,
                                              ctypes.c_float, ap_p, vp]
        L.glenside_pair_reduce.argtypes = [ap_p, ap_p, ctypes.c_int, ctypes.c_int, ap_p, vp]
        L.glenside_transpose.argtypes = [ap_p, i64_p, ap_p, vp]
        L.glenside_slice.argtypes = [ap_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ap_p, vp]
        L.glenside_concat.argtypes = [ap_p, ap_p, ctypes.c_int, ap_p, vp]
        L.glenside_pad.argtypes = [ap_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ap_p, vp]
        L.glenside_pair.argtypes = [ap_p, ap_p, ap_p, vp]
        L.glenside_cartesian_dot_blocked.argtypes = [ap_p, ap_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ap_p, vp]
        L.glenside_depthwise_conv2d.argtypes = [ap_p, ap_p, i64_p, i64_p, ctypes.c_int, ap_p, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().glenside_status_string(int(status)).decode()


def make_ap(t: Optional[torch.Tensor], n_access: int, shape: Optional[Sequence[int]] = None) -> gs_ap:
    """Descriptor for a contiguous tensor viewed with `n_access` access dimensions.

    `shape` overrides the tensor's own shape (same element count): flatten / reshape / squeeze of
    dense row-major data change the descriptor only.
    """
    ap = gs_ap()
    if not t.is_contiguous():
        raise ValueError("access patterns are dense row-major tensors")
    dims = tuple(t.shape) if shape is None else tuple(int(s) for s in shape)
    if len(dims) > GS_MAX_RANK:
        raise ValueError("rank above GS_MAX_RANK")
    ap.data = t.data_ptr()
    ap.dtype = _DTYPES[t.dtype]
    ap.rank = len(dims)
    ap.n_access = int(n_access)
    ap.reserved = 0
    for i, s in enumerate(dims):
        ap.shape[i] = int(s)
    return ap


def _i64(values: Optional[Sequence[int]]):
    if values is None:
        return None
    return (ctypes.c_int64 * len(values))(*[int(v) for v in values])


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream if t.is_cuda else 0


def _check(status: int, where: str) -> None:
    if status != GS_OK:
        raise GlensideError(status, where)


def windows_out_shape(in_shape: Sequence[int], n_access: int, window, stride, pad_lo=None, pad_hi=None):
    """Shape rule of `windows`: returns (shape tuple, n_access) of the result."""
    a = gs_ap()
    a.dtype, a.rank, a.n_access = GS_F32, len(in_shape), n_access
    for i, s in enumerate(in_shape):
        a.shape[i] = int(s)
    out = gs_ap()
    _check(lib().glenside_windows_out_shape(ctypes.byref(a), _i64(window), _i64(stride), _i64(pad_lo),
                                            _i64(pad_hi), ctypes.byref(out)), "windows_out_shape")
    return tuple(out.shape[i] for i in range(out.rank)), out.n_access


def access_windows(x: torch.Tensor, n_access: int, window, stride, pad_lo=None, pad_hi=None,
                   pad_mode: int = GS_PAD_ZERO, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """`windows` over the compute dims of (access x n_access); returns a tensor of shape S_A ++ b' ++ w."""
    shape, _ = windows_out_shape(x.shape, n_access, window, stride, pad_lo, pad_hi)
    if out is None:
        out = torch.empty(shape, dtype=x.dtype, device=x.device)
    o = make_ap(out, n_access + len(window))
    _check(lib().glenside_access_windows(ctypes.byref(make_ap(x, n_access)), _i64(window), _i64(stride),
                                         _i64(pad_lo), _i64(pad_hi), pad_mode, ctypes.byref(o),
                                         _stream(x)), "access_windows")
    return out


def cartesian_dot(a0: torch.Tensor, a1: torch.Tensor, n_access0: int = 1, n_access1: int = 1,
                  out_dtype: Optional[torch.dtype] = None, act: int = GS_ACT_NONE,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """compute dotProd (cartProd (access a0 n0) (access a1 n1)) -> tensor of shape S_A(a0) ++ S_A(a1)."""
    if out is None:
        if out_dtype is None:
            out_dtype = torch.int32 if a0.dtype == torch.int8 else torch.float32
        out = torch.empty(tuple(a0.shape[:n_access0]) + tuple(a1.shape[:n_access1]), dtype=out_dtype,
                          device=a0.device)
    _check(lib().glenside_cartesian_dot(ctypes.byref(make_ap(a0, n_access0)),
                                        ctypes.byref(make_ap(a1, n_access1)),
                                        ctypes.byref(make_ap(out, out.dim())), act, None, 0,
                                        _stream(a0)), "cartesian_dot")
    return out


def _conv(fn_name: str, ws_name: str, x, w, stride, pad, residual, act, out_dtype, out, workspace):
    L = lib()
    xa, wa = make_ap(x, 1), make_ap(w, 1)
    st, pd = _i64(stride), _i64(pad)
    need = getattr(L, ws_name)(ctypes.byref(xa), ctypes.byref(wa), st, pd)
    if out is None:
        if out_dtype is None:
            out_dtype = torch.int32 if x.dtype == torch.int8 else torch.float32
        # H', W' from the library's shape rule of `windows` (window (C,Kh,Kw), strides (1,Sh,Sw))
        shape, _ = windows_out_shape(x.shape, 1, (x.shape[1], w.shape[2], w.shape[3]), (1, stride[0], stride[1]),
                                     (0, pad[0], pad[1]), (0, pad[0], pad[1]))
        out = torch.empty((x.shape[0], w.shape[0], shape[2], shape[3]), dtype=out_dtype, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    res = ctypes.byref(make_ap(residual, residual.dim())) if residual is not None else None
    _check(getattr(L, fn_name)(ctypes.byref(xa), ctypes.byref(wa), st, pd, res, act,
                               ctypes.byref(make_ap(out, 4)), workspace.data_ptr(),
                               workspace.numel(), _stream(x)), fn_name)
    return out


def conv2d_workspace(x: torch.Tensor, w: torch.Tensor, stride, pad, form: str = "direct",
                     x_shape: Optional[Sequence[int]] = None) -> int:
    """Workspace bytes of a convolution call; `x_shape` sizes it for activations of another shape
    (and x's dtype) without needing such a tensor."""
    name = "glenside_conv2d_direct_workspace" if form == "direct" else "glenside_conv2d_im2col_workspace"
    return int(getattr(lib(), name)(ctypes.byref(make_ap(x, 1, shape=x_shape)), ctypes.byref(make_ap(w, 1)),
                                    _i64(stride), _i64(pad)))


def conv2d_direct(x, w, stride=(1, 1), pad=(0, 0), residual=None, act=GS_ACT_NONE, out_dtype=None,
                  out=None, workspace=None) -> torch.Tensor:
    """Fig. 2a with the windows formed on chip; x (N,C,H,W), w (O,C,Kh,Kw) -> (N,O,H',W')."""
    return _conv("glenside_conv2d_direct", "glenside_conv2d_direct_workspace", x, w, stride, pad,
                 residual, act, out_dtype, out, workspace)


def depthwise_conv2d(x, w, stride=(1, 1), pad=(0, 0), act=GS_ACT_NONE, out_dtype=None, out=None) -> torch.Tensor:
    """Every channel convolved with its own filter: x (N,C,H,W), w (C,Kh,Kw) -> (N,C,H',W')."""
    if out is None:
        if out_dtype is None:
            out_dtype = torch.int32 if x.dtype == torch.int8 else torch.float32
        shape, _ = windows_out_shape(x.shape, 2, (w.shape[1], w.shape[2]), tuple(stride), tuple(pad), tuple(pad))
        out = torch.empty(tuple(shape[:4]), dtype=out_dtype, device=x.device)
    _check(lib().glenside_depthwise_conv2d(ctypes.byref(make_ap(x, 1)), ctypes.byref(make_ap(w, 1)),
                                           _i64(stride), _i64(pad), act, ctypes.byref(make_ap(out, 4)),
                                           _stream(x)), "depthwise_conv2d")
    return out


def conv2d_direct_static(x, w, stride=(1, 1), pad=(0, 0), residual=None, act=GS_ACT_NONE, out_dtype=None,
                         out=None) -> torch.Tensor:
    """`conv2d_direct` on the library's fixed scratch array: no workspace, nothing allocated by the
    call (pass `out` to keep torch from allocating the result either)."""
    if out is None:
        if out_dtype is None:
            out_dtype = torch.int32 if x.dtype == torch.int8 else torch.float32
        shape, _ = windows_out_shape(x.shape, 1, (x.shape[1], w.shape[2], w.shape[3]), (1, stride[0], stride[1]),
                                     (0, pad[0], pad[1]), (0, pad[0], pad[1]))
        out = torch.empty((x.shape[0], w.shape[0], shape[2], shape[3]), dtype=out_dtype, device=x.device)
    res = ctypes.byref(make_ap(residual, residual.dim())) if residual is not None else None
    _check(lib().glenside_conv2d_direct_static(ctypes.byref(make_ap(x, 1)), ctypes.byref(make_ap(w, 1)),
                                               _i64(stride), _i64(pad), res, act,
                                               ctypes.byref(make_ap(out, 4)), _stream(x)),
           "conv2d_direct_static")
    return out


def conv2d_direct_static_limit() -> int:
    return int(lib().glenside_conv2d_direct_static_limit())


def conv2d_pack_weights(w: torch.Tensor, packed: Optional[torch.Tensor] = None,
                        for_input: Optional[tuple] = None) -> torch.Tensor:
    """Weights (O,C,Kh,Kw) -> the packed form `conv2d_direct_packed` reads (a uint8 buffer).

    `for_input` = (x, stride, pad) sizes a new buffer for that call (`conv2d_workspace`), which may
    include scratch behind the weights; without it the buffer holds the weights only.
    """
    L = lib()
    wa = make_ap(w, 1)
    if packed is None:
        if for_input is not None:
            x, stride, pad = for_input
            need = conv2d_workspace(x, w, stride, pad)
        else:
            fake_x = gs_ap()
            fake_x.dtype, fake_x.rank, fake_x.n_access = wa.dtype, 4, 1
            fake_x.shape[0], fake_x.shape[1], fake_x.shape[2], fake_x.shape[3] = 1, w.shape[1], w.shape[2], w.shape[3]
            need = L.glenside_conv2d_direct_workspace(ctypes.byref(fake_x), ctypes.byref(wa), _i64((1, 1)), _i64((0, 0)))
        packed = torch.empty(max(int(need), 16), dtype=torch.uint8, device=w.device)
    _check(L.glenside_conv2d_pack_weights(ctypes.byref(wa), packed.data_ptr(), packed.numel(), _stream(w)),
           "conv2d_pack_weights")
    return packed


def conv2d_direct_packed(x, w, packed, stride=(1, 1), pad=(0, 0), residual=None, act=GS_ACT_NONE,
                         out_dtype=None, out=None) -> torch.Tensor:
    """Fig. 2a reading weights from `conv2d_pack_weights(w)`; `w` supplies shape and dtype only."""
    return _conv("glenside_conv2d_direct_packed", "glenside_conv2d_direct_workspace", x, w, stride, pad,
                 residual, act, out_dtype, out, packed)


def conv2d_im2col(x, w, stride=(1, 1), pad=(0, 0), residual=None, act=GS_ACT_NONE, out_dtype=None,
                  out=None, workspace=None) -> torch.Tensor:
    """Fig. 5: explicit flatten(windows) in the workspace, then the dense contraction."""
    return _conv("glenside_conv2d_im2col", "glenside_conv2d_im2col_workspace", x, w, stride, pad,
                 residual, act, out_dtype, out, workspace)


def _reduce_out_dtype(x: torch.Tensor, op: int, out_dtype):
    if out_dtype is not None:
        return out_dtype
    if x.dtype == torch.int8:
        return torch.int32 if op == GS_SUM else torch.int8
    return x.dtype


def reduce(x: torch.Tensor, n_access: int, op: int, scale: float = 1.0, out_dtype=None,
           out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """compute reduceSum|reduceMax (access x n_access) -> tensor of shape S_A."""
    if out is None:
        out = torch.empty(tuple(x.shape[:n_access]), dtype=_reduce_out_dtype(x, op, out_dtype),
                          device=x.device)
    _check(lib().glenside_reduce(ctypes.byref(make_ap(x, n_access)), op, scale,
                                 ctypes.byref(make_ap(out, out.dim())), _stream(x)), "reduce")
    return out


def windows_reduce(x: torch.Tensor, n_access: int, window, stride, pad_lo=None, pad_hi=None,
                   op: int = GS_MAX, scale: float = 1.0, out_dtype=None,
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """compute reduce (windows (access x n_access) window stride) without materialising the windows."""
    if out is None:
        shape, na = windows_out_shape(x.shape, n_access, window, stride, pad_lo, pad_hi)
        out = torch.empty(shape[:na], dtype=_reduce_out_dtype(x, op, out_dtype), device=x.device)
    _check(lib().glenside_windows_reduce(ctypes.byref(make_ap(x, n_access)), _i64(window), _i64(stride),
                                         _i64(pad_lo), _i64(pad_hi), op, scale,
                                         ctypes.byref(make_ap(out, out.dim())), _stream(x)),
           "windows_reduce")
    return out


def pair_reduce(a: torch.Tensor, b: torch.Tensor, op: int = GS_SUM, act: int = GS_ACT_NONE,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """compute reduceSum|reduceMax (pair a b) for patterns with empty compute shape: element-wise."""
    if out is None:
        out = torch.empty_like(a)
    _check(lib().glenside_pair_reduce(ctypes.byref(make_ap(a, a.dim())), ctypes.byref(make_ap(b, b.dim())),
                                      op, act, ctypes.byref(make_ap(out, out.dim())), _stream(a)),
           "pair_reduce")
    return out


def transpose(x: torch.Tensor, n_access: int, perm: Sequence[int],
              out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """transpose (access x n_access) perm, materialised: output dimension t is input dimension perm[t]."""
    if out is None:
        out = torch.empty([x.shape[p] for p in perm], dtype=x.dtype, device=x.device)
    _check(lib().glenside_transpose(ctypes.byref(make_ap(x, n_access)), _i64(perm),
                                    ctypes.byref(make_ap(out, n_access)), _stream(x)), "transpose")
    return out


def slice_(x: torch.Tensor, n_access: int, dim: int, lo: int, hi: int,
           out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """slice (access x n_access) dim lo hi, materialised."""
    if out is None:
        shape = list(x.shape)
        shape[dim] = hi - lo
        out = torch.empty(shape, dtype=x.dtype, device=x.device)
    _check(lib().glenside_slice(ctypes.byref(make_ap(x, n_access)), dim, lo, hi,
                                ctypes.byref(make_ap(out, n_access)), _stream(x)), "slice")
    return out


def concat(a: torch.Tensor, b: torch.Tensor, n_access: int, dim: int,
           out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """concat a b dim, materialised."""
    if out is None:
        shape = list(a.shape)
        shape[dim] = a.shape[dim] + b.shape[dim]
        out = torch.empty(shape, dtype=a.dtype, device=a.device)
    _check(lib().glenside_concat(ctypes.byref(make_ap(a, n_access)), ctypes.byref(make_ap(b, n_access)), dim,
                                 ctypes.byref(make_ap(out, n_access)), _stream(a)), "concat")
    return out


def pad(x: torch.Tensor, n_access: int, dim: int, lo: int, hi: int, pad_mode: int = GS_PAD_ZERO,
        out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """EXT pad: dimension dim grows by lo cells in front and hi behind."""
    if out is None:
        shape = list(x.shape)
        shape[dim] = x.shape[dim] + lo + hi
        out = torch.empty(shape, dtype=x.dtype, device=x.device)
    _check(lib().glenside_pad(ctypes.byref(make_ap(x, n_access)), dim, lo, hi, pad_mode,
                              ctypes.byref(make_ap(out, n_access)), _stream(x)), "pad")
    return out


def pair(a: torch.Tensor, b: torch.Tensor, n_access: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """pair a b: ((a..),(c..)) x 2 -> ((a..),(2, c..)), materialised."""
    if out is None:
        shape = list(a.shape[:n_access]) + [2] + list(a.shape[n_access:])
        out = torch.empty(shape, dtype=a.dtype, device=a.device)
    _check(lib().glenside_pair(ctypes.byref(make_ap(a, n_access)), ctypes.byref(make_ap(b, n_access)),
                               ctypes.byref(make_ap(out, n_access)), _stream(a)), "pair")
    return out


def cartesian_dot_blocked(a0: torch.Tensor, a1: torch.Tensor, tile_m: int, tile_n: int, tile_k: int,
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The blocked form of compute dotProd (cartProd a0 a1) for matrices ((M),(K)) x ((N),(K))."""
    if out is None:
        out_dtype = torch.int32 if a0.dtype == torch.int8 else torch.float32
        out = torch.empty((a0.shape[0], a1.shape[0]), dtype=out_dtype, device=a0.device)
    _check(lib().glenside_cartesian_dot_blocked(ctypes.byref(make_ap(a0, 1)), ctypes.byref(make_ap(a1, 1)),
                                                tile_m, tile_n, tile_k, ctypes.byref(make_ap(out, 2)),
                                                _stream(a0)), "cartesian_dot_blocked")
    return out


# ---------------------------------------------------------------------------------------------
# programs as text
# ---------------------------------------------------------------------------------------------

_META_DTYPES = {v: k for k, v in _DTYPES.items()}


def _named(tensors, ints):
    """Marshal {name: tensor or (shape, dtype)} and {name: int}; returns the arrays and what keeps them alive."""
    keep = []
    ta = (gs_named_ap * max(len(tensors), 1))()
    for i, (name, t) in enumerate(tensors.items()):
        nb = name.encode()
        keep.append(nb)
        ta[i].name = nb
        if isinstance(t, torch.Tensor):
            ta[i].tensor = make_ap(t, 0)
        else:                                   # shape and dtype only (host-side queries)
            shape, dtype = t
            ap = gs_ap()
            ap.dtype, ap.rank = _DTYPES[dtype], len(shape)
            for d, v in enumerate(shape):
                ap.shape[d] = int(v)
            ta[i].tensor = ap
    ia = (gs_named_int * max(len(ints), 1))()
    for i, (name, v) in enumerate(ints.items()):
        nb = name.encode()
        keep.append(nb)
        ia[i].name = nb
        ia[i].value = int(v)
    return ta, len(tensors), ia, len(ints), keep


def program_shape(text: str, tensors, ints=None):
    """Shape rule of a whole program: returns (shape tuple, n_access, torch dtype)."""
    ta, nt, ia, ni, _keep = _named(tensors, ints or {})
    out = gs_ap()
    _check(lib().glenside_program_shape(text.encode(), ta, nt, ia, ni, ctypes.byref(out)), "program_shape")
    return tuple(out.shape[i] for i in range(out.rank)), out.n_access, _META_DTYPES[out.dtype]


def program_eval(text: str, tensors, ints=None, out_dtype=None, out: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Evaluate an access-pattern program (the paper's s-expression text) on the GPU."""
    ints = ints or {}
    ta, nt, ia, ni, _keep = _named(tensors, ints)
    L = lib()
    shape, na, dtype = program_shape(text, tensors, ints)
    first = next(iter(tensors.values()))
    if out is None:
        out = torch.empty(shape, dtype=out_dtype or dtype, device=first.device)
    if workspace is None:
        need = L.glenside_program_workspace(text.encode(), ta, nt, ia, ni)
        workspace = torch.empty(max(int(need), 16), dtype=torch.uint8, device=first.device)
    _check(L.glenside_program_eval(text.encode(), ta, nt, ia, ni, ctypes.byref(make_ap(out, na, shape=shape)),
                                   workspace.data_ptr(), workspace.numel(), _stream(first)), "program_eval")
    return out


def program_rewrite(text: str, strategy: str, tensors, ints=None, params: Sequence[int] = ()) -> str:
    """Apply the paper's rewrite rules ("im2col", "systolic", "block" with params (bm, bn, bk))."""
    ta, nt, ia, ni, _keep = _named(tensors, ints or {})
    L = lib()
    need = ctypes.c_size_t(0)
    st = L.glenside_program_rewrite(text.encode(), strategy.encode(), _i64(params) if params else None,
                                    len(params), ta, nt, ia, ni, None, 0, ctypes.byref(need))
    if st != GS_ERR_WORKSPACE:
        _check(st, "program_rewrite")
    buf = ctypes.create_string_buffer(need.value)
    _check(L.glenside_program_rewrite(text.encode(), strategy.encode(), _i64(params) if params else None,
                                      len(params), ta, nt, ia, ni, buf, need.value, None), "program_rewrite")
    return buf.value.decode()
