"""GPU parity of programs given as text: the same s-expression goes to the CPU oracle's interpreter
and to `glenside_program_eval`; integer results bit-exact, bfloat16 within 1e-2 relative."""

import numpy as np
import pytest
import torch

from oracle import sexpr
from paper_2105_09377_amd import binding as gs, synth
from helpers import assert_parity, fp8_slack, to_oracle
import listings

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_both(text, tensors, ints=None, out_dtype=None):
    ints = ints or {}
    want = sexpr.evaluate(text, {k: to_oracle(v) for k, v in tensors.items()}, ints)
    got = gs.program_eval(text, {k: v.to(DEV) for k, v in tensors.items()}, ints, out_dtype=out_dtype)
    assert tuple(got.shape) == want.shape
    return got, want


@pytest.mark.parametrize("dtype,odt", [("i8", None), ("bf16", None), ("bf16", torch.bfloat16)])
@pytest.mark.parametrize("shape", [(2, 3, 9, 8, 5, 3, 2, 2, 1), (3, 64, 20, 20, 70, 3, 3, 1, 1), (2, 16, 12, 12, 8, 1, 1, 2, 2)])
def test_conv2d_listing(dtype, odt, shape):
    n, c, h, w, o, kh, kw, sh, sw = shape
    cfg = synth.conv_layer(n, c, h, w, o, kh, 1, 0, dtype, 9300 + c + o)
    wt = cfg["w"][:, :, :, :kw].contiguous()
    ints = dict(C=c, Kh=kh, Kw=kw, Sh=sh, Sw=sw)
    tensors = {"activations": cfg["x"], "weights": wt}
    got, want = run_both(listings.CONV2D, tensors, ints, odt)
    assert_parity(got, want.materialize(), what=f"Fig. 2a {dtype} {shape}")
    # the program the im2col rules derive from it (Fig. 5), evaluated node by node: explicit
    # windows -> flatten -> contraction -> reshape -> squeeze -> transpose
    meta = {k: (tuple(v.shape), v.dtype) for k, v in tensors.items()}
    im2col = gs.program_rewrite(listings.CONV2D, "im2col", meta, ints)
    got2 = gs.program_eval(im2col, {k: v.to(DEV) for k, v in tensors.items()}, ints, out_dtype=odt)
    assert_parity(got2, want.materialize(), what=f"Fig. 5 {dtype} {shape}")
    if dtype == "i8":
        assert torch.equal(got, got2)


def test_conv2d_listing_on_padded_tensor():
    cfg = synth.conv_layer(2, 32, 14, 14, 40, 3, 1, 1, "i8", 9400)
    ints = dict(C=32, Kh=3, Kw=3, Sh=1, Sw=1, Ph=1, Pw=1)
    got, want = run_both(listings.CONV2D_PADDED, {"activations": cfg["x"], "weights": cfg["w"]}, ints)
    assert_parity(got, want.materialize(), what="padded Fig. 2a")
    assert torch.equal(got, gs.conv2d_direct(cfg["x"].to(DEV), cfg["w"].to(DEV), (1, 1), (1, 1)))


@pytest.mark.parametrize("dtype", ["i8", "bf16", "fp8"])
@pytest.mark.parametrize("dims", [(32, 32, 32), (70, 96, 200)])
def test_matmul_listing_and_its_rewrites(dtype, dims):
    m, n, k = dims
    if dtype == "i8":
        a, w = synth.uniform_int8((m, k), -127, 127, 9500), synth.uniform_int8((k, n), -127, 127, 9501)
    elif dtype == "bf16":
        a, w = synth.normal_bf16((m, k), 1.0, 9500), synth.normal_bf16((k, n), k ** -0.5, 9501)
    else:
        a, w = synth.normal_fp8((m, k), 1.0, 9500), synth.normal_fp8((k, n), k ** -0.5, 9501)
    tensors = {"activations": a, "weights": w}
    got, want = run_both(listings.MATMUL, tensors)
    ref = want.materialize()
    slack = fp8_slack(to_oracle(a), to_oracle(w).T) if dtype == "fp8" else None
    assert_parity(got, ref, what="Fig. 2b", slack=slack)
    meta = {k_: (tuple(v.shape), v.dtype) for k_, v in tensors.items()}
    dev = {k_: v.to(DEV) for k_, v in tensors.items()}
    blocked = gs.program_rewrite(listings.MATMUL, "block", meta, params=(16, 32, 16))
    assert_parity(gs.program_eval(blocked, dev), ref, what="blocked program (Fig. 7)", slack=slack)
    systolic = gs.program_rewrite(listings.MATMUL, "systolic", meta)
    assert_parity(gs.program_eval(systolic, dev), ref, what="systolicArray (Fig. 3)", slack=slack)


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f32"])
def test_maxpool_listing(dtype):
    x = {"i8": synth.uniform_int8((3, 5, 17, 18), -127, 127, 9600), "bf16": synth.normal_bf16((3, 5, 17, 18), 1.0, 9600),
         "f32": synth.normal_f32((3, 5, 17, 18), 1.0, 9600)}[dtype]
    got, want = run_both(listings.MAXPOOL, {"activations": x}, dict(Kh=3, Kw=2, Sh=2, Sw=2))
    np.testing.assert_array_equal(to_oracle(got), want.materialize())


def test_transformer_compositions():
    a = synth.normal_f32((6, 10), 1.0, 9700)
    b = synth.normal_f32((6, 10), 1.0, 9701)
    t = {"a": a, "b": b}
    for text in [
        "(compute reduceSum (pair (access a 2) (access b 2)))",                       # element-wise sum (Sec. 5.4)
        "(compute reduceMax (pair (access a 2) (access b 2)))",
        "(compute reduceSum (access a 1))",
        "(compute reduceSum (pair (access a 1) (access b 1)))",                       # folds the rows as well
        "(concat (slice (access a 1) 1 0 4) (slice (access b 1) 1 4 10) 1)",
        "(transpose (concat (access a 1) (access b 1) 0) (list 1 0))",
        "(slice (access a 1) 0 2 5)",                                                 # a view, copied out
        "(access a 1)",
        "(flatten (pair (access a 1) (access b 1)))",
        "(compute relu (compute reduceSum (pair (access a 2) (access b 2))))",
        "(reshape (compute reduceSum (windows (access a 1) (shape 4) (shape 3))) (shape 3 6) (shape))",
    ]:
        got, want = run_both(text, t)
        assert_parity(got, want.materialize(), float_tol=1e-5, what=text)


def test_unsupported_and_workspace_errors():
    a = synth.normal_bf16((8, 16), 1.0, 9800).to(DEV)
    with pytest.raises(gs.GlensideError) as e:
        gs.program_eval("(cartProd (access a 1) (access a 1))", {"a": a})            # a bare Cartesian product
    assert e.value.status == gs.GS_ERR_UNSUPPORTED
    out = torch.empty((8, 8), dtype=torch.float32, device=DEV)
    with pytest.raises(gs.GlensideError) as e:
        gs.program_eval("(compute dotProd (cartProd (access a 1) (slice (access a 1) 1 0 16)))", {"a": a}, out=out,
                        workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.status == gs.GS_ERR_WORKSPACE


@pytest.mark.parametrize("dtype", ["i8", "bf16"])
def test_random_programs(dtype):
    """Two hundred seeded random programs (Table 1 transformers, dotProd / reduceSum / reduceMax) on small
    tensors: whatever the library accepts must equal the oracle -- bit for bit on int8 inputs -- and it must
    accept most of them; what it refuses, it must refuse with a status, launching nothing."""
    import random_programs
    rng = np.random.default_rng(20210509 + (0 if dtype == "i8" else 1))
    shapes = {"a": (3, 4, 6, 5), "b": (6, 8), "c": (2, 1, 7)}
    def make(shape, stream):
        return synth.uniform_int8(shape, -5, 5, stream) if dtype == "i8" else synth.normal_bf16(shape, 1.0, stream)
    tensors = {k: make(s, 9900 + i) for i, (k, s) in enumerate(shapes.items())}
    tensors.update({k + "2": make(s, 9950 + i) for i, (k, s) in enumerate(shapes.items())})
    same = {k: (k[:-1] if k.endswith("2") else k + "2") for k in tensors}
    host = {k: to_oracle(v) for k, v in tensors.items()}
    dev = {k: v.to(DEV) for k, v in tensors.items()}
    ran = refused = 0
    for i in range(200):
        text = random_programs.grow(rng, host, same, depth=int(rng.integers(1, 6)))
        want = sexpr.evaluate(text, host)
        try:
            got = gs.program_eval(text, dev)
        except gs.GlensideError as e:
            # rank: a cartProd inside a dotProd may exceed the eight dimensions of the boundary
            assert e.status in (gs.GS_ERR_UNSUPPORTED, gs.GS_ERR_DTYPE) or \
                (e.status == gs.GS_ERR_RANK and "cartProd" in text), (text, e.status)
            refused += 1
            continue
        ran += 1
        assert tuple(got.shape) == want.shape, text
        ref = want.materialize()
        if not np.isfinite(ref.astype(np.float64)).all():        # reduceMax over a padded window of -inf etc.
            np.testing.assert_array_equal(np.isfinite(to_oracle(got)), np.isfinite(ref), err_msg=text)
            continue
        # a chain of computes stores its intermediate results in bfloat16 (one more rounding of
        # 2^-9 per link, which a later cancellation can amplify); the oracle keeps fp64 throughout
        chained = dtype == "bf16" and text.count("compute") > 1
        assert_parity(got, ref, float_tol=5e-2 if chained else 1e-2, what=text)
    assert ran >= 150, (ran, refused)
