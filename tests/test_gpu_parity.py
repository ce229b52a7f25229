"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded inputs.

Integer results must be bit-exact; bf16-in / fp32-accumulate results must be within 1e-2 maximum
relative error (floor 1e-3 * max|ref| on the denominator).  Sizes span several tiles and ragged
tails of the kernels' 32/64/128-wide tiles.
"""

import numpy as np
import pytest
import torch

from oracle import access_pattern as ap
from oracle import brute
from oracle import programs as pg
from paper_2105_09377_amd import binding as gs
from paper_2105_09377_amd import synth
from helpers import assert_parity, fp8_slack, to_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gen(dtype, shape, stream, scale=1.0):
    if dtype == "i8":
        return synth.uniform_int8(shape, -127, 127, stream)
    if dtype == "i32":
        return synth.uniform_int32(shape, -100000, 100000, stream)
    if dtype == "bf16":
        return synth.normal_bf16(shape, scale, stream)
    if dtype == "fp8":
        return synth.normal_fp8(shape, scale, stream)
    return synth.normal_f32(shape, scale, stream)


def oracle_windows(x, n_access, window, stride, pad_lo, pad_hi, fill):
    node = ap.tensor(to_oracle(x))
    nc = x.dim() - n_access
    for d in range(nc):
        lo = pad_lo[d] if pad_lo else 0
        hi = pad_hi[d] if pad_hi else 0
        if lo or hi:
            node = ap.pad(node, n_access + d, lo, hi, fill)
    return ap.windows(ap.access(node, n_access), window, stride)


LOWEST = {"i8": -128, "i32": -2 ** 31, "bf16": -np.inf, "f32": -np.inf}

# ---------------------------------------------------------------------------------------------
# windows
# ---------------------------------------------------------------------------------------------

WINDOW_CASES = [
    # dtype, shape, n_access, window, stride, pad_lo, pad_hi, pad_mode
    ("f32", (5, 37), 1, (4,), (3,), None, None, gs.GS_PAD_ZERO),
    ("bf16", (2, 3, 9, 11), 2, (3, 2), (2, 3), (1, 0), (1, 1), gs.GS_PAD_LOWEST),
    ("i8", (1, 3, 8, 8), 1, (3, 3, 3), (1, 1, 1), None, None, gs.GS_PAD_ZERO),
    ("i8", (2, 5, 13, 10), 1, (5, 3, 3), (1, 2, 2), (0, 1, 1), (0, 1, 1), gs.GS_PAD_ZERO),
    ("bf16", (3, 16, 20, 20), 1, (16, 3, 3), (1, 1, 1), (0, 1, 1), (0, 1, 1), gs.GS_PAD_ZERO),
    ("i32", (2, 2, 6, 7), 2, (2, 2), (2, 2), None, None, gs.GS_PAD_LOWEST),
    ("bf16", (2, 3, 15, 15), 1, (3, 7, 7), (1, 2, 2), (0, 3, 3), (0, 3, 3), gs.GS_PAD_ZERO),
    # convolution-shaped windows through LDS: 16-byte rows, several channel passes, strides,
    # asymmetric padding, every element size
    ("bf16", (2, 8, 24, 32), 1, (8, 3, 3), (1, 1, 1), (0, 1, 1), (0, 1, 1), gs.GS_PAD_ZERO),
    ("bf16", (1, 320, 6, 40), 1, (320, 3, 3), (1, 1, 1), (0, 1, 1), (0, 1, 1), gs.GS_PAD_ZERO),
    ("i8", (2, 48, 10, 48), 1, (48, 3, 3), (1, 2, 2), (0, 1, 1), (0, 1, 1), gs.GS_PAD_LOWEST),
    ("i8", (1, 16, 9, 21), 1, (16, 2, 4), (1, 1, 3), (0, 0, 2), (0, 1, 0), gs.GS_PAD_ZERO),
    ("f32", (3, 4, 11, 12), 1, (4, 5, 3), (1, 2, 1), (0, 2, 1), (0, 2, 1), gs.GS_PAD_LOWEST),
    ("i32", (1, 8, 7, 9), 1, (8, 1, 1), (1, 2, 2), None, None, gs.GS_PAD_ZERO),
]


@pytest.mark.parametrize("case", WINDOW_CASES)
def test_access_windows(case):
    dtype, shape, na, window, stride, lo, hi, mode = case
    x = gen(dtype, shape, 1000 + len(shape) + shape[-1])
    got = gs.access_windows(x.to(DEV), na, window, stride, lo, hi, mode)
    fill = LOWEST[dtype] if mode == gs.GS_PAD_LOWEST else 0
    want = oracle_windows(x, na, window, stride, lo, hi, fill).materialize()
    got_np = to_oracle(got)
    assert got_np.shape == want.shape
    np.testing.assert_array_equal(got_np, want)          # a gather is exact in every dtype


def test_access_windows_is_the_im2col_matrix():
    """flatten(windows ...) of Fig. 5 is the same memory as the windows result."""
    x = gen("i8", (2, 4, 9, 9), 1100)
    got = gs.access_windows(x.to(DEV), 1, (4, 3, 3), (1, 2, 2), (0, 1, 1), (0, 1, 1))
    want = pg.im2col_matrix(ap.tensor(to_oracle(x)), (4, 3, 3), (2, 2), (1, 1)).materialize()
    np.testing.assert_array_equal(to_oracle(got).reshape(want.shape), want)


# ---------------------------------------------------------------------------------------------
# compute dotProd (cartProd a0 a1)
# ---------------------------------------------------------------------------------------------

DOT_CASES = [
    # dtype, a0 shape, n0, a1 shape, n1, out dtype, relu
    ("i8", (36, 27), 1, (4, 27), 1, torch.int32, False),          # the tiny conv's im2col product
    ("i8", (300, 328), 1, (200, 328), 1, torch.int32, False),     # ragged tiles, K not a slab multiple
    ("i8", (130, 1000), 1, (70, 1000), 1, torch.int32, True),
    ("bf16", (256, 784), 1, (512, 784), 1, torch.float32, True),  # MLP layer 1
    ("bf16", (256, 512), 1, (10, 512), 1, torch.float32, False),  # MLP layer 3
    ("bf16", (100, 147), 1, (64, 147), 1, torch.bfloat16, False), # K = 147: unaligned rows
    ("bf16", (2, 3, 4, 5), 2, (7, 4, 5), 1, torch.float32, False),  # multi-dim access and compute shapes
    ("bf16", (513, 64), 1, (129, 64), 1, torch.bfloat16, True),
    ("i8", (1, 5), 1, (1, 5), 1, torch.int32, False),
    # K a whole number of 32-byte steps but not of 128-byte slabs: short last slab
    ("bf16", (70, 80), 1, (300, 80), 1, torch.float32, False),
    ("bf16", (33, 16), 1, (65, 16), 1, torch.bfloat16, True),
    ("i8", (129, 96), 1, (140, 96), 1, torch.int32, False),
    ("bf16", (300, 784), 1, (512, 784), 1, torch.bfloat16, True),
    # result rows written 8 and 4 columns per lane, in every result type
    ("i8", (64, 128), 1, (72, 128), 1, torch.int32, True),
    ("bf16", (40, 64), 1, (76, 64), 1, torch.bfloat16, False),
    ("bf16", (200, 256), 1, (264, 256), 1, torch.float32, False),
    # 8-bit floats: 64-byte K steps; K not a multiple of 64 takes the checked kernel
    ("fp8", (300, 328), 1, (200, 328), 1, torch.float32, False),
    ("fp8", (130, 1000), 1, (70, 1000), 1, torch.bfloat16, True),
    ("fp8", (64, 128), 1, (72, 128), 1, torch.float32, True),
    ("fp8", (129, 192), 1, (140, 192), 1, torch.bfloat16, False),   # short last slab
    ("fp8", (2, 3, 4, 8), 2, (7, 4, 8), 1, torch.float32, False),
    ("fp8", (1, 5), 1, (1, 5), 1, torch.float32, False),
    ("fp8", (256, 832), 1, (512, 832), 1, torch.float32, True),
]


@pytest.mark.parametrize("case", DOT_CASES)
def test_cartesian_dot(case):
    dtype, s0, n0, s1, n1, odt, relu = case
    k = int(np.prod(s0[n0:]))
    a0 = gen(dtype, s0, 1200 + s0[0], 1.0)
    a1 = gen(dtype, s1, 1300 + s1[0], 1.0 / np.sqrt(k) if dtype in ("bf16", "fp8") else 1.0)
    got = gs.cartesian_dot(a0.to(DEV), a1.to(DEV), n0, n1, odt, gs.GS_ACT_RELU if relu else gs.GS_ACT_NONE)
    prog = pg.cartesian_dot(ap.access(ap.tensor(to_oracle(a0)), n0), ap.access(ap.tensor(to_oracle(a1)), n1))
    if relu:
        prog = ap.compute(ap.relu, prog)
    assert tuple(got.shape) == prog.access_shape
    slack = None
    if dtype == "fp8":
        slack = fp8_slack(to_oracle(a0).reshape(-1, k), to_oracle(a1).reshape(-1, k)).reshape(prog.access_shape)
    assert_parity(got, prog.materialize(), what=str(case), slack=slack)


def test_cartesian_dot_extreme_int8_values():
    """-128 * -128 * K stays exact in int32."""
    a0 = torch.full((40, 512), -128, dtype=torch.int8)
    a1 = torch.full((33, 512), -128, dtype=torch.int8)
    got = gs.cartesian_dot(a0.to(DEV), a1.to(DEV))
    assert (got.cpu() == 128 * 128 * 512).all()


def test_cartesian_dot_fp8_every_code():
    """All 254 finite e4m3 codes (subnormals, -0, +-448) as operands: the hardware must read the
    OCP encoding (bias 7, no infinities), not a variant with another bias or NaN placement."""
    codes = np.arange(256, dtype=np.uint8)
    codes[codes == 0x7F] = 0
    codes[codes == 0xFF] = 0x80
    a0 = torch.from_numpy(np.stack([np.roll(codes, r) for r in range(64)])).view(torch.float8_e4m3fn)
    a1 = gen("fp8", (40, 256), 1777, 0.5)
    for odt in (torch.float32, torch.bfloat16):
        got = gs.cartesian_dot(a0.to(DEV), a1.to(DEV), 1, 1, odt)
        assert_parity(got, brute.matmul(to_oracle(a0), to_oracle(a1).T), float_tol=1e-2, what=str(odt),
                      slack=fp8_slack(to_oracle(a0), to_oracle(a1)))
    # one code at a time against 1.0: the products are the decoded values themselves
    eye = torch.from_numpy(np.where(np.eye(256, dtype=bool), 0x38, 0).astype(np.uint8)).view(torch.float8_e4m3fn)
    row = torch.from_numpy(np.tile(codes, (3, 1))).view(torch.float8_e4m3fn)
    got = gs.cartesian_dot(row.to(DEV), eye.to(DEV), 1, 1, torch.float32).cpu().numpy().astype(np.float64)
    np.testing.assert_array_equal(got, np.tile(to_oracle(row)[0], (3, 1)))


def test_cartesian_dot_empty():
    a0 = torch.zeros((0, 16), dtype=torch.bfloat16, device=DEV)
    a1 = torch.zeros((8, 16), dtype=torch.bfloat16, device=DEV)
    assert gs.cartesian_dot(a0, a1).shape == (0, 8)

# Products large enough for the 256x256 (8 waves) and 128x128 tiles of the direct-to-LDS kernel,
# with ragged last tiles in both directions and results written 8, 4 and 1 columns per lane.
# Sampled rows of a0 (first, last, and both sides of tile boundaries) against every row of a1.
BIG_DOT_CASES = [
    # dtype, I, J, K, out dtype, relu
    ("bf16", 4100, 4104, 512, torch.bfloat16, True),     # 256x256, 8 columns per lane
    ("bf16", 4100, 4100, 512, torch.float32, False),     # 256x256, 4 columns per lane
    ("bf16", 4099, 4099, 144, torch.bfloat16, False),    # 256x256, one column per lane, short last slab
    ("i8", 4100, 4104, 512, torch.int32, True),          # 256x256 int8
    ("i8", 4100, 4099, 96, torch.int32, False),
    ("bf16", 1800, 1808, 264 * 2, torch.bfloat16, True), # 128x128, 8 columns per lane
    ("bf16", 1800, 1804, 264 * 2, torch.float32, False), # 128x128, 4 columns per lane
    ("i8", 1801, 1803, 160, torch.int32, False),         # 128x128, one column per lane
    ("i8", 1800, 1808, 512, torch.int32, True),
    ("fp8", 4100, 4104, 512, torch.bfloat16, True),      # 256x256, 8-bit floats
    ("fp8", 4100, 4099, 192, torch.float32, False),      # short last slab
    ("fp8", 1800, 1804, 576, torch.float32, False),      # 128x128
]


@pytest.mark.parametrize("case", BIG_DOT_CASES)
def test_cartesian_dot_large_tiles(case):
    dtype, I, J, K, odt, relu = case
    a0 = gen(dtype, (I, K), 1400 + I + K, 1.0)
    a1 = gen(dtype, (J, K), 1500 + J + K, 1.0 / np.sqrt(K) if dtype in ("bf16", "fp8") else 1.0)
    got = gs.cartesian_dot(a0.to(DEV), a1.to(DEV), 1, 1, odt, gs.GS_ACT_RELU if relu else gs.GS_ACT_NONE)
    rows = sorted({0, 1, 31, 32, 63, 64, 127, 128, 129, 255, 256, 257, 1023, 1024, I // 2, I - 130, I - 5, I - 2, I - 1}
                  | set(int(v) for v in np.random.default_rng(I + J).integers(0, I, 40)))
    idx = torch.tensor(rows)
    want = brute.matmul(to_oracle(a0[idx]), to_oracle(a1).T)
    if relu:
        want = np.maximum(want, 0)
    slack = fp8_slack(to_oracle(a0[idx]), to_oracle(a1)) if dtype == "fp8" else None
    assert_parity(got[idx.to(DEV)], want, what=str(case), slack=slack)


@pytest.mark.parametrize("dtype,odt", [("bf16", torch.bfloat16), ("bf16", torch.float32), ("i8", torch.int32)])
@pytest.mark.parametrize("o,n", [(256, 21), (128, 8), (192, 24)])
def test_conv2d_im2col_large_tiles_residual_relu(dtype, odt, o, n):
    """1x1 convolutions whose im2col product takes the 256x256 (O = 256, 65856 positions; O = 192
    with a ragged channel tile) and 128x128 (O = 128, 25088 positions) tiles, with the fused
    residual and ReLU and the (N,O,H',W') addressing of the stores; whole images."""
    cfg = synth.conv_layer(n, 64, 56, 56, o, 1, 1, 0, dtype, 8100 + o + n, gain=1.0)
    res = gen("i32" if dtype == "i8" else ("bf16" if odt == torch.bfloat16 else "f32"), (n, o, 56, 56), 8200 + o)
    got = gs.conv2d_im2col(cfg["x"].to(DEV), cfg["w"].to(DEV), (1, 1), (0, 0), residual=res.to(DEV),
                           act=gs.GS_ACT_RELU, out_dtype=odt)
    idx = torch.tensor([0, n // 2, n - 1])
    want = brute.conv2d(to_oracle(cfg["x"][idx]), to_oracle(cfg["w"]), (1, 1), (0, 0)) + to_oracle(res[idx])
    assert_parity(got[idx.to(DEV)], np.maximum(want, 0), what=f"{dtype} O={o} N={n}")



# ---------------------------------------------------------------------------------------------
# conv2d, both forms
# ---------------------------------------------------------------------------------------------

CONV_CASES = [
    # dtype, N, C, H, W, O, Kh, Kw, stride, pad, out dtype
    ("i8", 1, 3, 8, 8, 4, 3, 3, (1, 1), (0, 0), torch.int32),          # tiny configuration
    ("i8", 3, 40, 13, 13, 70, 3, 3, (1, 1), (1, 1), torch.int32),       # odd W, ragged C / O / M tails
    ("i8", 2, 64, 20, 18, 33, 3, 3, (2, 2), (1, 1), torch.int32),
    ("bf16", 2, 16, 20, 20, 24, 3, 3, (1, 1), (1, 1), torch.float32),
    ("bf16", 5, 32, 7, 7, 130, 3, 3, (1, 1), (1, 1), torch.bfloat16),   # 49-position planes: tiles span images
    ("bf16", 3, 24, 14, 14, 48, 1, 1, (2, 2), (0, 0), torch.float32),   # 1x1 stride-2 projection
    ("bf16", 2, 3, 30, 30, 16, 7, 7, (2, 2), (3, 3), torch.bfloat16),   # 7x7/2 pad 3, C = 3
    ("bf16", 1, 48, 9, 11, 20, 3, 2, (1, 2), (0, 1), torch.float32),    # non-square everything
    ("bf16", 2, 128, 12, 12, 64, 3, 3, (1, 1), (1, 1), torch.float32),  # several channel chunks
    # fewer channels than a 32-byte chunk: im2col rows formed in LDS (conv_smallc)
    ("bf16", 2, 1, 19, 23, 5, 3, 3, (1, 1), (1, 1), torch.float32),      # odd width: scalar staging
    ("bf16", 1, 3, 40, 272, 70, 5, 3, (2, 1), (2, 1), torch.bfloat16),   # two channel tiles, Wo > 128
    ("bf16", 2, 8, 16, 16, 64, 3, 3, (1, 1), (1, 1), torch.bfloat16),
    ("i8", 2, 16, 12, 32, 33, 3, 3, (1, 2), (1, 1), torch.int32),
    ("i8", 1, 3, 9, 9, 4, 1, 1, (1, 1), (0, 0), torch.int32),
    # few channels, windows a whole number of dwords apart: fragments read straight from the staged rows
    ("bf16", 2, 3, 33, 37, 20, 5, 8, (1, 2), (2, 3), torch.float32),     # 8-wide kernel rows
    ("bf16", 1, 2, 20, 300, 70, 3, 3, (2, 2), (1, 1), torch.bfloat16),   # Wo = 150, two channel tiles
    ("i8", 2, 4, 16, 40, 33, 3, 5, (1, 4), (1, 2), torch.int32),
    ("bf16", 3, 1, 9, 9, 4, 1, 1, (2, 2), (0, 0), torch.float32),
    # few output tiles, many chunks: the channel sum is split among workgroups (2 and 4 ways)
    ("bf16", 2, 256, 7, 7, 128, 3, 3, (1, 1), (1, 1), torch.bfloat16),
    ("bf16", 3, 128, 8, 8, 96, 3, 3, (1, 1), (1, 1), torch.float32),
    ("i8", 2, 512, 7, 7, 64, 3, 3, (1, 1), (1, 1), torch.int32),
    ("bf16", 2, 256, 14, 14, 64, 1, 1, (2, 2), (0, 0), torch.bfloat16),
    # odd widths: rows moved as runs of four pixels that cross row ends, unaligned loads
    ("bf16", 3, 64, 9, 7, 70, 3, 3, (1, 1), (1, 1), torch.bfloat16),
    ("bf16", 2, 64, 15, 13, 64, 3, 3, (2, 2), (1, 1), torch.float32),
    ("bf16", 7, 64, 7, 7, 32, 5, 5, (1, 1), (2, 2), torch.float32),
    ("bf16", 1, 64, 33, 45, 48, 3, 3, (1, 1), (0, 0), torch.bfloat16),
    ("i8", 2, 128, 7, 9, 33, 3, 3, (1, 1), (1, 1), torch.int32),
]


def conv_inputs(case):
    dtype, n, c, h, w, o, kh, kw, stride, pad, odt = case
    x = gen(dtype, (n, c, h, w), 1400 + c + h)
    wt = gen(dtype, (o, c, kh, kw), 1500 + o, 1.0 / np.sqrt(c * kh * kw) if dtype == "bf16" else 1.0)
    return x, wt


def conv_oracle(x, wt, stride, pad):
    xo, wo = to_oracle(x), to_oracle(wt)
    macs = x.shape[0] * wt.shape[0] * x.shape[2] * x.shape[3] * wt[0].numel()
    if macs <= 4_000_000:
        return pg.conv2d(ap.tensor(xo), ap.tensor(wo), stride, pad).materialize()
    return brute.conv2d(xo, wo, stride, pad)


@pytest.mark.parametrize("form", ["direct", "im2col"])
@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d(case, form):
    x, wt = conv_inputs(case)
    stride, pad, odt = case[8], case[9], case[10]
    fn = gs.conv2d_direct if form == "direct" else gs.conv2d_im2col
    got = fn(x.to(DEV), wt.to(DEV), stride, pad, out_dtype=odt)
    assert_parity(got, conv_oracle(x, wt, stride, pad), what=f"{form} {case}")


def _random_conv_cases(seed, count):
    """Seeded shapes across the kernels' branches: channel counts on and off the 16 / 32 multiples,
    widths that are and are not multiples of the producers' vectors, planes of 7..40, strides,
    paddings up to half the window, rectangular windows, few and many output channels."""
    r = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        dtype = ("bf16", "i8")[int(r.integers(2))]
        n = int(r.integers(1, 6))
        c = int(r.choice([3, 8, 16, 24, 32, 48, 64, 96, 128, 160, 256]))
        h, w = int(r.integers(5, 41)), int(r.integers(5, 41))
        o = int(r.choice([1, 5, 32, 64, 70, 128, 200, 256]))
        kh, kw = [(1, 1), (3, 3), (3, 3), (3, 3), (5, 5), (3, 2), (2, 3)][int(r.integers(7))]
        stride = (int(r.integers(1, 3)), int(r.integers(1, 3)))
        pad = (int(r.integers(0, kh // 2 + 1)), int(r.integers(0, kw // 2 + 1)))
        if h + 2 * pad[0] < kh or w + 2 * pad[1] < kw or n * c * h * w * o * kh * kw > 3e9:
            continue
        odt = torch.int32 if dtype == "i8" else (torch.bfloat16, torch.float32)[int(r.integers(2))]
        cases.append((dtype, n, c, h, w, o, kh, kw, stride, pad, odt, bool(r.integers(2)), bool(r.integers(2))))
    return cases


@pytest.mark.parametrize("case", _random_conv_cases(20210905, 48))
def test_conv2d_random_shapes(case):
    """Both forms on seeded random shapes, with and without the fused residual and ReLU."""
    dtype, n, c, h, w, o, kh, kw, stride, pad, odt, with_res, relu = case
    x, wt = conv_inputs(case[:11])
    ho, wo_ = (h + 2 * pad[0] - kh) // stride[0] + 1, (w + 2 * pad[1] - kw) // stride[1] + 1
    res = None
    if with_res:
        res = (synth.uniform_int32((n, o, ho, wo_), -50000, 50000, 1701) if odt == torch.int32 else
               synth.normal_bf16((n, o, ho, wo_), 1.0, 1702) if odt == torch.bfloat16 else
               synth.normal_f32((n, o, ho, wo_), 1.0, 1703))
    want = brute.conv2d(to_oracle(x), to_oracle(wt), stride, pad)
    if res is not None:
        want = want + to_oracle(res)
    if relu:
        want = np.maximum(want, 0)
    act = gs.GS_ACT_RELU if relu else gs.GS_ACT_NONE
    outs = []
    for fn in (gs.conv2d_direct, gs.conv2d_im2col):
        got = fn(x.to(DEV), wt.to(DEV), stride, pad, residual=None if res is None else res.to(DEV), act=act, out_dtype=odt)
        assert_parity(got, want, what=f"{fn.__name__} {case}")
        outs.append(got)
    if dtype == "i8":
        assert torch.equal(outs[0], outs[1])


def test_conv2d_direct_equals_im2col_bitwise_int8():
    """The rewrite of Sec. 5.3 preserves the result: both forms agree bit for bit on integers."""
    case = ("i8", 4, 32, 17, 19, 40, 3, 3, (1, 1), (1, 1), torch.int32)
    x, wt = conv_inputs(case)
    a = gs.conv2d_direct(x.to(DEV), wt.to(DEV), (1, 1), (1, 1))
    b = gs.conv2d_im2col(x.to(DEV), wt.to(DEV), (1, 1), (1, 1))
    assert torch.equal(a, b)
    assert_parity(a, conv_oracle(x, wt, (1, 1), (1, 1)))


@pytest.mark.parametrize("form", ["direct", "im2col"])
@pytest.mark.parametrize("hw", [10, 12, 9])    # planes of 100, 144, 81 positions: 4, 8, 1 results per store
@pytest.mark.parametrize("c", [32, 128])     # 128 channels: enough chunks for the producer / consumer kernel
@pytest.mark.parametrize("dtype,odt", [("i8", torch.int32), ("bf16", torch.bfloat16), ("bf16", torch.float32)])
def test_conv2d_residual_relu(form, dtype, odt, hw, c):
    case = (dtype, 2, c, hw, hw, 40, 3, 3, (1, 1), (1, 1), odt)
    x, wt = conv_inputs(case)
    if odt == torch.int32:
        res = synth.uniform_int32((2, 40, hw, hw), -50000, 50000, 1601)
    elif odt == torch.bfloat16:
        res = synth.normal_bf16((2, 40, hw, hw), 1.0, 1602)
    else:
        res = synth.normal_f32((2, 40, hw, hw), 1.0, 1603)
    fn = gs.conv2d_direct if form == "direct" else gs.conv2d_im2col
    got = fn(x.to(DEV), wt.to(DEV), (1, 1), (1, 1), residual=res.to(DEV), act=gs.GS_ACT_RELU, out_dtype=odt)
    conv = pg.conv2d(ap.tensor(to_oracle(x)), ap.tensor(to_oracle(wt)), (1, 1), (1, 1))
    prog = ap.compute(ap.relu, pg.add(conv, ap.access(ap.tensor(to_oracle(res)), 4)))
    assert_parity(got, prog.materialize(), what=f"{form} {dtype} residual+relu")


@pytest.mark.parametrize("dtype,odt,hw", [("bf16", torch.bfloat16, 7), ("bf16", torch.float32, 8), ("i8", torch.int32, 8)])
def test_conv2d_split_channel_sum_residual_relu(dtype, odt, hw):
    """Split channel sums are combined with the residual and ReLU in a second kernel; and the
    packed entry point gives the same result with and without the scratch that enables the split."""
    c = 512 if dtype == "i8" else 256
    case = (dtype, 2, c, hw, hw, 128, 3, 3, (1, 1), (1, 1), odt)
    x, wt = conv_inputs(case)
    shape = (2, 128, hw, hw)
    res = {torch.int32: lambda: synth.uniform_int32(shape, -50000, 50000, 1611),
           torch.bfloat16: lambda: synth.normal_bf16(shape, 1.0, 1612),
           torch.float32: lambda: synth.normal_f32(shape, 1.0, 1613)}[odt]()
    xd, wd, rd = x.to(DEV), wt.to(DEV), res.to(DEV)
    assert gs.conv2d_workspace(xd, wd, (1, 1), (1, 1)) > gs.conv2d_pack_weights(wd).numel()   # scratch is asked for
    got = gs.conv2d_direct(xd, wd, (1, 1), (1, 1), residual=rd, act=gs.GS_ACT_RELU, out_dtype=odt)
    want = np.maximum(brute.conv2d(to_oracle(x), to_oracle(wt), (1, 1), (1, 1)) + to_oracle(res), 0)
    assert_parity(got, want, what="split")
    plain = gs.conv2d_direct_packed(xd, wd, gs.conv2d_pack_weights(wd), (1, 1), (1, 1), residual=rd,
                                    act=gs.GS_ACT_RELU, out_dtype=odt)
    assert_parity(plain, want, what="unsplit")


@pytest.mark.parametrize("odt", [torch.bfloat16, torch.float32])
def test_conv2d_few_channels_residual_relu(odt):
    case = ("bf16", 2, 3, 20, 24, 40, 7, 7, (2, 2), (3, 3), odt)
    x, wt = conv_inputs(case)
    shape = (2, 40, 10, 12)
    res = synth.normal_bf16(shape, 1.0, 1621) if odt == torch.bfloat16 else synth.normal_f32(shape, 1.0, 1622)
    got = gs.conv2d_direct(x.to(DEV), wt.to(DEV), (2, 2), (3, 3), residual=res.to(DEV), act=gs.GS_ACT_RELU, out_dtype=odt)
    want = np.maximum(brute.conv2d(to_oracle(x), to_oracle(wt), (2, 2), (3, 3)) + to_oracle(res), 0)
    assert_parity(got, want, what="few channels, residual + relu")


def _random_few_channel_cases(seed, count):
    """Seeded shapes for the few-channel kernel: 1..4 channels (8 for int8), windows of 3..7, rows
    that are and are not whole 16-byte vectors, output heights on and off the multiples of four
    (a task is four output rows), output widths on and off the multiples of 4 and 8 and past 128."""
    r = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        dtype = ("bf16", "bf16", "i8")[int(r.integers(3))]
        n = int(r.integers(1, 4))
        c = int(r.integers(1, 5)) if dtype == "bf16" else int(r.choice([1, 3, 4, 8]))
        h = int(r.integers(7, 60))
        w = int(r.choice([8, 16, 24, 31, 32, 40, 50, 56, 64, 100, 160, 272]))
        o = int(r.choice([5, 32, 64, 70]))
        k = int(r.choice([3, 5, 7]))
        stride = (int(r.integers(1, 3)), int(r.integers(1, 3)))
        pad = (int(r.integers(0, k // 2 + 1)), int(r.integers(0, k // 2 + 1)))
        if h + 2 * pad[0] < k or w + 2 * pad[1] < k:
            continue
        odt = torch.int32 if dtype == "i8" else (torch.bfloat16, torch.float32)[int(r.integers(2))]
        cases.append((dtype, n, c, h, w, o, k, k, stride, pad, odt, bool(r.integers(2)), bool(r.integers(2))))
    return cases


@pytest.mark.parametrize("case", _random_few_channel_cases(20210908, 40))
def test_conv2d_few_channels_random_shapes(case):
    dtype, n, c, h, w, o, kh, kw, stride, pad, odt, with_res, relu = case
    x, wt = conv_inputs(case[:11])
    ho, wo_ = (h + 2 * pad[0] - kh) // stride[0] + 1, (w + 2 * pad[1] - kw) // stride[1] + 1
    res = None
    if with_res:
        res = (synth.uniform_int32((n, o, ho, wo_), -50000, 50000, 1711) if odt == torch.int32 else
               synth.normal_bf16((n, o, ho, wo_), 1.0, 1712) if odt == torch.bfloat16 else
               synth.normal_f32((n, o, ho, wo_), 1.0, 1713))
    want = brute.conv2d(to_oracle(x), to_oracle(wt), stride, pad)
    if res is not None:
        want = want + to_oracle(res)
    if relu:
        want = np.maximum(want, 0)
    got = gs.conv2d_direct(x.to(DEV), wt.to(DEV), stride, pad, residual=None if res is None else res.to(DEV),
                           act=gs.GS_ACT_RELU if relu else gs.GS_ACT_NONE, out_dtype=odt)
    assert_parity(got, want, what=str(case))


def test_conv2d_minus_128_and_empty_batch():
    x = torch.full((1, 32, 6, 6), -128, dtype=torch.int8)
    w = torch.full((8, 32, 3, 3), -128, dtype=torch.int8)
    got = gs.conv2d_direct(x.to(DEV), w.to(DEV), (1, 1), (1, 1))
    assert_parity(got, conv_oracle(x, w, (1, 1), (1, 1)))
    empty = torch.zeros((0, 32, 6, 6), dtype=torch.int8, device=DEV)
    assert gs.conv2d_direct(empty, w.to(DEV), (1, 1), (1, 1)).shape == (0, 8, 6, 6)
    assert gs.conv2d_im2col(empty, w.to(DEV), (1, 1), (1, 1)).shape == (0, 8, 6, 6)


# ---------------------------------------------------------------------------------------------
# reduce, pooling, pair
# ---------------------------------------------------------------------------------------------

REDUCE_CASES = [
    ("i8", (7, 13), 1), ("i8", (3, 5, 4), 1), ("i32", (10, 49), 1), ("bf16", (6, 5, 7, 7), 2),
    ("f32", (33, 100), 1), ("bf16", (3, 5000), 1), ("f32", (1000, 1), 1), ("i32", (2, 9000), 1),
    ("bf16", (513, 4), 1), ("f32", (5,), 0),
    # many short rows: staged through LDS, 128 rows per workgroup, ragged last workgroup
    ("bf16", (600, 49), 1), ("i8", (777, 33), 1), ("f32", (515, 9), 1), ("i32", (1030, 13), 1),
    ("bf16", (9, 64, 7, 7), 2),
]


@pytest.mark.parametrize("op", [gs.GS_SUM, gs.GS_MAX])
@pytest.mark.parametrize("case", REDUCE_CASES)
def test_reduce(case, op):
    dtype, shape, na = case
    x = gen(dtype, shape, 1700 + len(shape) + shape[0])
    got = gs.reduce(x.to(DEV), na, op)
    oper = ap.reduceSum if op == gs.GS_SUM else ap.reduceMax
    want = ap.compute(oper, ap.access(ap.tensor(to_oracle(x)), na)).materialize()
    if op == gs.GS_MAX:
        np.testing.assert_array_equal(to_oracle(got), want)      # max is exact in every dtype
    else:
        assert_parity(got, want, float_tol=1e-2 if dtype == "bf16" else 1e-4, what=str(case))


def test_reduce_scaled_mean_is_global_average_pool():
    x = gen("bf16", (4, 24, 7, 7), 1801)
    got = gs.reduce(x.to(DEV), 2, gs.GS_SUM, scale=1.0 / 49.0)
    prog = ap.compute(ap.scale(1.0 / 49.0), ap.compute(ap.reduceSum, ap.access(ap.tensor(to_oracle(x)), 2)))
    assert_parity(got, prog.materialize())


POOL_CASES = [
    ("bf16", (2, 5, 14, 14), (2, 2), (2, 2), None),
    ("bf16", (2, 3, 17, 16), (3, 3), (2, 2), (1, 1)),
    ("i8", (1, 4, 9, 12), (3, 2), (1, 2), (1, 0)),
    ("f32", (2, 2, 8, 8), (8, 8), (1, 1), None),
    ("i32", (3, 3, 10, 10), (2, 2), (2, 2), None),
    ("bf16", (3, 4, 112, 112), (3, 3), (2, 2), (1, 1)),     # the ResNet stem pooling plane
    ("bf16", (1, 2, 150, 136), (3, 3), (2, 2), (1, 1)),     # several bands of rows per plane
    ("f32", (1, 3, 70, 200), (5, 3), (3, 2), (2, 1)),       # run-time window, several bands
    ("i8", (2, 3, 33, 64), (2, 2), (2, 2), None),
    ("i8", (1, 2, 31, 35), (3, 3), (1, 1), (1, 1)),
]


@pytest.mark.parametrize("case", POOL_CASES)
def test_max_pool_fused_and_unfused(case):
    dtype, shape, window, stride, pad = case
    x = gen(dtype, shape, 1900 + shape[-1])
    xd = x.to(DEV)
    fused = gs.windows_reduce(xd, 2, window, stride, pad, pad, gs.GS_MAX)
    win = gs.access_windows(xd, 2, window, stride, pad, pad, gs.GS_PAD_LOWEST)
    unfused = gs.reduce(win, 4, gs.GS_MAX)
    want = pg.max_pool2d(ap.tensor(to_oracle(x)), window, stride, pad or (0, 0), LOWEST[dtype]).materialize()
    np.testing.assert_array_equal(to_oracle(fused), want)
    assert torch.equal(fused, unfused)


def test_sum_pool_and_1d_windows_reduce():
    x = gen("f32", (3, 40), 1950)
    got = gs.windows_reduce(x.to(DEV), 1, (5,), (3,), (2,), (2,), gs.GS_SUM, scale=0.2)
    node = ap.windows(ap.access(ap.pad(ap.tensor(to_oracle(x)), 1, 2, 2, 0.0), 1), (5,), (3,))
    want = ap.compute(ap.scale(0.2), ap.compute(ap.reduceSum, node)).materialize()
    assert_parity(got, want, float_tol=1e-5)


SUM_POOL_CASES = [
    ("bf16", (2, 6, 7, 7), (7, 7), (1, 1), None, 1.0 / 49.0, torch.float32),
    ("bf16", (2, 3, 40, 48), (3, 3), (2, 2), (1, 1), 1.0 / 9.0, torch.bfloat16),
    ("i8", (2, 3, 12, 16), (2, 2), (2, 2), None, 1.0, torch.int32),
    ("f32", (1, 2, 90, 100), (4, 4), (4, 4), None, 0.0625, torch.float32),
]


@pytest.mark.parametrize("case", SUM_POOL_CASES)
def test_sum_pool_2d(case):
    dtype, shape, window, stride, pad, scale, odt = case
    x = gen(dtype, shape, 1960 + shape[-1])
    got = gs.windows_reduce(x.to(DEV), 2, window, stride, pad, pad, gs.GS_SUM, scale=scale, out_dtype=odt)
    node = ap.tensor(to_oracle(x))
    if pad:
        node = ap.pad(ap.pad(node, 2, pad[0], pad[0], 0), 3, pad[1], pad[1], 0)
    prog = ap.compute(ap.reduceSum, ap.windows(ap.access(node, 2), window, stride))
    if scale != 1.0:
        prog = ap.compute(ap.scale(scale), prog)
    # fp32 accumulation of up to 49 terms against an fp64 sum: error <= 49 * 2^-24 * sum|x|, and the
    # result may be 1e-3 of that sum after cancellation (the floor in rel_error) -> 1e-4 covers it.
    assert_parity(got, prog.materialize(), float_tol=1e-2 if odt == torch.bfloat16 else 1e-4)


@pytest.mark.parametrize("dtype", ["i32", "bf16", "f32"])
@pytest.mark.parametrize("op", [gs.GS_SUM, gs.GS_MAX])
def test_pair_reduce(dtype, op):
    a, b = gen(dtype, (3, 5, 7, 11), 2001), gen(dtype, (3, 5, 7, 11), 2002)
    got = gs.pair_reduce(a.to(DEV), b.to(DEV), op, gs.GS_ACT_RELU)
    oper = ap.reduceSum if op == gs.GS_SUM else ap.reduceMax
    pr = ap.pair(ap.access(ap.tensor(to_oracle(a)), 4), ap.access(ap.tensor(to_oracle(b)), 4))
    want = ap.compute(ap.relu, ap.compute(oper, pr)).materialize()
    assert_parity(got, want, float_tol=1e-2 if dtype == "bf16" else 1e-6)


# ---------------------------------------------------------------------------------------------
# transformers that move data: transpose, slice, concat, pair, pad
# ---------------------------------------------------------------------------------------------

def assert_same_values(got, node, what):
    """A transformer only moves elements: the stored values must be the oracle's, exactly."""
    want = node.materialize()
    assert tuple(got.shape) == tuple(want.shape), what
    np.testing.assert_array_equal(to_oracle(got), want, err_msg=what)


TRANSPOSE_CASES = [
    # dtype, shape, n_access, perm
    ("bf16", (3, 20, 20, 24), 1, (0, 3, 1, 2)),      # the (N,H',W',O) -> (N,O,H',W') tail of Fig. 5
    ("f32", (70, 130), 1, (1, 0)),                   # ((N),(O)) -> ((O),(N)), ragged 64 x 64 tiles
    ("i8", (5, 67, 33), 2, (0, 2, 1)),
    ("i32", (4, 3, 5, 6), 2, (3, 1, 0, 2)),          # no dimension keeps its place
    ("bf16", (6, 7, 64), 1, (1, 0, 2)),              # the contiguous dimension stays: rows are copied
    ("bf16", (2, 3, 4, 5, 6), 3, (4, 3, 2, 1, 0)),
    ("f32", (9,), 1, (0,)),
    ("i8", (2, 64, 136), 1, (0, 2, 1)),              # 8 elements per lane
    ("bf16", (3, 7, 9), 1, (0, 2, 1)),               # odd extents: one element per lane
]


@pytest.mark.parametrize("case", TRANSPOSE_CASES)
def test_transpose(case):
    dtype, shape, na, perm = case
    x = gen(dtype, shape, 2100 + len(shape) + shape[0])
    got = gs.transpose(x.to(DEV), na, perm)
    assert_same_values(got, ap.transpose(ap.access(ap.tensor(to_oracle(x)), na), perm), str(case))


SLICE_CASES = [
    ("bf16", (4, 64, 40), 1, 1, 8, 56), ("i8", (37, 19), 1, 1, 3, 17), ("f32", (10, 6, 8), 2, 0, 2, 9),
    ("i32", (5, 12), 1, 1, 4, 4), ("bf16", (3, 5, 7, 16), 2, 2, 1, 6),
]


@pytest.mark.parametrize("case", SLICE_CASES)
def test_slice(case):
    dtype, shape, na, dim, lo, hi = case
    x = gen(dtype, shape, 2200 + shape[0])
    got = gs.slice_(x.to(DEV), na, dim, lo, hi)
    assert_same_values(got, ap.slice_(ap.access(ap.tensor(to_oracle(x)), na), dim, lo, hi), str(case))


CONCAT_CASES = [
    ("bf16", (4, 24, 32), (4, 40, 32), 1, 1), ("i8", (3, 5), (3, 9), 1, 1), ("f32", (2, 6, 8), (5, 6, 8), 1, 0),
    ("i32", (4, 3, 0), (4, 3, 5), 2, 2), ("bf16", (2, 3, 4, 8), (2, 3, 4, 24), 2, 3),
]


@pytest.mark.parametrize("case", CONCAT_CASES)
def test_concat(case):
    dtype, sa, sb, na, dim = case
    a, b = gen(dtype, sa, 2300 + sa[0]), gen(dtype, sb, 2310 + sb[0])
    got = gs.concat(a.to(DEV), b.to(DEV), na, dim)
    node = ap.concat(ap.access(ap.tensor(to_oracle(a)), na), ap.access(ap.tensor(to_oracle(b)), na), dim)
    assert_same_values(got, node, str(case))


@pytest.mark.parametrize("case", [("bf16", (6, 5, 16), 1), ("i8", (7, 3), 1), ("f32", (4, 9, 2), 2),
                                  ("i32", (5, 8), 2), ("bf16", (33, 64), 0)])
def test_pair(case):
    dtype, shape, na = case
    a, b = gen(dtype, shape, 2400 + shape[0]), gen(dtype, shape, 2410 + shape[0])
    got = gs.pair(a.to(DEV), b.to(DEV), na)
    node = ap.pair(ap.access(ap.tensor(to_oracle(a)), na), ap.access(ap.tensor(to_oracle(b)), na))
    assert_same_values(got, node, str(case))


@pytest.mark.parametrize("case", [("bf16", (3, 8, 16), 1, 2, 8, 8, gs.GS_PAD_ZERO), ("i8", (5, 7), 1, 1, 2, 3, gs.GS_PAD_LOWEST),
                                  ("f32", (4, 6, 5), 2, 1, 1, 0, gs.GS_PAD_LOWEST), ("i32", (2, 9), 1, 0, 0, 0, gs.GS_PAD_ZERO)])
def test_pad(case):
    dtype, shape, na, dim, lo, hi, mode = case
    x = gen(dtype, shape, 2500 + shape[0])
    got = gs.pad(x.to(DEV), na, dim, lo, hi, mode)
    fill = LOWEST[dtype] if mode == gs.GS_PAD_LOWEST else 0
    assert_same_values(got, ap.pad(ap.access(ap.tensor(to_oracle(x)), na), dim, lo, hi, fill), str(case))


@pytest.mark.parametrize("dtype,block", [("i8", 16), ("i8", 32), ("bf16", 16), ("bf16", 64)])
def test_cartesian_dot_blocked_is_the_blocked_program(dtype, block):
    """Square blocks, every dimension a multiple: the program of Fig. 7 generalised, block by block."""
    m, k, o = 2 * block, 4 * block, 3 * block
    a = gen(dtype, (m, k), 2701 + block, 1.0)
    w = gen(dtype, (k, o), 2702 + block, 1.0 / np.sqrt(k) if dtype == "bf16" else 1.0)    # (K,O) as in Fig. 2b
    wt = gs.transpose(w.to(DEV), 1, (1, 0))                                                 # ((O),(K))
    got = gs.cartesian_dot_blocked(a.to(DEV), wt, block, block, block)
    prog, count = pg.blocked_matmul(ap.tensor(to_oracle(a)), ap.tensor(to_oracle(w)), block)
    assert count == 2 * 3 * 4
    assert_parity(got, prog.materialize(), what=f"blocked {dtype} {block}")
    if dtype == "i8":
        assert torch.equal(got, gs.cartesian_dot(a.to(DEV), wt))


@pytest.mark.parametrize("tiles", [(64, 64, 128), (100, 48, 80), (1000, 1000, 1000), (17, 256, 33),
                                   (100, 48, 128), (17, 200, 64), (128, 130, 256), (150, 64, 64)])
def test_cartesian_dot_blocked_ragged_tiles(tiles):
    """Tile sizes that do not divide the matrix: last blocks and last K slices are smaller."""
    a0, a1 = gen("i8", (150, 328), 2801), gen("i8", (130, 328), 2802)
    got = gs.cartesian_dot_blocked(a0.to(DEV), a1.to(DEV), *tiles)
    assert torch.equal(got, gs.cartesian_dot(a0.to(DEV), a1.to(DEV)))
    b0, b1 = gen("bf16", (150, 320), 2803), gen("bf16", (130, 320), 2804, 1.0 / np.sqrt(320))
    gotf = gs.cartesian_dot_blocked(b0.to(DEV), b1.to(DEV), *tiles)
    prog = pg.cartesian_dot(ap.access(ap.tensor(to_oracle(b0)), 1), ap.access(ap.tensor(to_oracle(b1)), 1))
    assert_parity(gotf, prog.materialize(), what=f"ragged {tiles}")
    c0, c1 = gen("fp8", (150, 320), 2805), gen("fp8", (130, 320), 2806, 1.0 / np.sqrt(320))
    got8 = gs.cartesian_dot_blocked(c0.to(DEV), c1.to(DEV), *tiles)
    assert_parity(got8, brute.matmul(to_oracle(c0), to_oracle(c1).T), what=f"ragged fp8 {tiles}",
                  slack=fp8_slack(to_oracle(c0), to_oracle(c1)))


@pytest.mark.parametrize("dtype,tiles", [("bf16", (512, 512, 128)), ("i8", (512, 768, 256)), ("fp8", (1024, 512, 128)),
                                         ("bf16", (384, 640, 64))])
def test_cartesian_dot_blocked_one_launch_large(dtype, tiles):
    """Blocks large enough for the 256x256 and 128x128 tiles, a last block of four rows, K slices that
    are whole slabs (one launch); sampled rows on both sides of block boundaries against the oracle."""
    I, J, K = 4100, 4104, 256
    a0 = gen(dtype, (I, K), 2901, 1.0)
    a1 = gen(dtype, (J, K), 2902, 1.0 / np.sqrt(K) if dtype != "i8" else 1.0)
    got = gs.cartesian_dot_blocked(a0.to(DEV), a1.to(DEV), *tiles)
    bm = tiles[0]
    rows = sorted({0, 1, 255, 256, bm - 1, bm, bm + 1, 2 * bm - 1, 2 * bm, I - 5, I - 4, I - 3, I - 1}
                  | set(int(v) for v in np.random.default_rng(7).integers(0, I, 30)))
    idx = torch.tensor(rows)
    want = brute.matmul(to_oracle(a0[idx]), to_oracle(a1).T)
    assert_parity(got[idx.to(DEV)], want, what=f"{dtype} {tiles}",
                  slack=fp8_slack(to_oracle(a0[idx]), to_oracle(a1)) if dtype == "fp8" else None)
    if dtype == "i8":
        assert torch.equal(got, gs.cartesian_dot(a0.to(DEV), a1.to(DEV)))


def test_blocked_matmul_from_slices_and_concat():
    """Fig. 7 on the GPU: a matmul split in two along N and K with slice, cartProd/dotProd on the
    blocks, pair + reduceSum over the K halves and concat along N equals the unblocked product
    (exactly, for integers)."""
    a = gen("i8", (48, 128), 2601)
    b = gen("i8", (80, 128), 2602)
    A, B = a.to(DEV), b.to(DEV)
    whole = gs.cartesian_dot(A, B)
    cols = []
    for n0, n1 in ((0, 32), (32, 80)):
        bn = gs.slice_(B, 1, 0, n0, n1)
        halves = [gs.cartesian_dot(gs.slice_(A, 1, 1, k0, k0 + 64), gs.slice_(bn, 1, 1, k0, k0 + 64)) for k0 in (0, 64)]
        cols.append(gs.pair_reduce(halves[0], halves[1], gs.GS_SUM))
    blocked = gs.concat(cols[0], cols[1], 2, 1)
    assert torch.equal(blocked, whole)
    prog = pg.cartesian_dot(ap.access(ap.tensor(to_oracle(a)), 1), ap.access(ap.tensor(to_oracle(b)), 1))
    assert_parity(blocked, prog.materialize(), what="blocked matmul")


# ---------------------------------------------------------------------------------------------
# depth-wise windows
# ---------------------------------------------------------------------------------------------

def oracle_depthwise(x, w, stride, pad):
    """C one-channel convolutions (brute-force loops), stacked along the channel dimension."""
    xo, wo = to_oracle(x), to_oracle(w)
    return np.concatenate([brute.conv2d(np.ascontiguousarray(xo[:, c:c + 1]), np.ascontiguousarray(wo[c:c + 1, None]),
                                        stride, pad) for c in range(x.shape[1])], axis=1)


def test_depthwise_is_the_sliced_program():
    """Small case against the program itself: slice / Fig. 2a / concat, evaluated by the interpreter."""
    for dtype, odt in (("bf16", torch.float32), ("i8", torch.int32)):
        x, w = gen(dtype, (2, 5, 9, 11), 3101), gen(dtype, (5, 3, 3), 3102, 0.3)
        got = gs.depthwise_conv2d(x.to(DEV), w.to(DEV), (1, 1), (1, 1), out_dtype=odt)
        prog = pg.depthwise_conv2d(ap.tensor(to_oracle(x)), ap.tensor(to_oracle(w)[:, None]), (1, 1), (1, 1))
        assert tuple(got.shape) == prog.access_shape
        assert_parity(got, prog.materialize(), what=f"depth-wise program {dtype}")


DEPTHWISE_CASES = [
    # dtype, N, C, H, W, Kh, Kw, stride, pad, out dtype, relu
    ("bf16", 3, 24, 56, 56, 3, 3, (1, 1), (1, 1), torch.bfloat16, False),   # several planes per task, 16-byte stores
    ("bf16", 2, 16, 112, 112, 3, 3, (2, 2), (1, 1), torch.bfloat16, True),  # one plane per task, stride 2
    ("bf16", 1, 3, 300, 200, 3, 3, (1, 1), (1, 1), torch.float32, False),   # planes cut into bands of rows
    ("bf16", 1, 2, 301, 203, 3, 3, (2, 2), (1, 1), torch.bfloat16, False),  # bands, stride 2, odd sizes
    ("bf16", 4, 40, 14, 14, 3, 3, (1, 1), (1, 1), torch.bfloat16, True),    # rows that are no multiple of 16 bytes
    ("bf16", 5, 67, 7, 7, 3, 3, (1, 1), (1, 1), torch.float32, False),      # ragged last group of planes
    ("bf16", 2, 6, 28, 28, 3, 3, (2, 2), (1, 1), torch.bfloat16, False),
    ("bf16", 2, 7, 13, 17, 5, 5, (1, 1), (2, 2), torch.float32, True),      # 5x5
    ("bf16", 2, 3, 20, 19, 3, 2, (2, 1), (1, 0), torch.float32, False),     # run-time window loops
    ("bf16", 2, 3, 9, 9, 1, 1, (1, 1), (0, 0), torch.bfloat16, False),      # 1x1: a per-channel scale
    ("bf16", 1, 1, 3, 3, 3, 3, (1, 1), (0, 0), torch.float32, False),       # a single window
    ("i8", 3, 24, 56, 56, 3, 3, (1, 1), (1, 1), torch.int32, False),
    ("i8", 2, 9, 112, 112, 3, 3, (2, 2), (1, 1), torch.int32, True),
    ("i8", 4, 33, 14, 14, 3, 3, (1, 1), (1, 1), torch.int32, False),
    ("i8", 1, 2, 200, 333, 5, 5, (1, 1), (2, 2), torch.int32, False),
    ("i8", 2, 3, 20, 19, 4, 3, (3, 2), (0, 2), torch.int32, False),
]


@pytest.mark.parametrize("case", DEPTHWISE_CASES)
def test_depthwise_conv2d(case):
    dtype, n, c, h, w_, kh, kw, stride, pad, odt, relu = case
    x = gen(dtype, (n, c, h, w_), 3200 + c + h)
    w = gen(dtype, (c, kh, kw), 3300 + c + kh, 1.0 / np.sqrt(kh * kw) if dtype == "bf16" else 1.0)
    got = gs.depthwise_conv2d(x.to(DEV), w.to(DEV), stride, pad, gs.GS_ACT_RELU if relu else gs.GS_ACT_NONE, odt)
    want = oracle_depthwise(x, w, stride, pad)
    if relu:
        want = np.maximum(want, 0)
    assert_parity(got, want, what=str(case))


def test_depthwise_extremes_and_empty():
    x = torch.full((2, 3, 10, 10), -128, dtype=torch.int8)
    w = torch.full((3, 3, 3), -128, dtype=torch.int8)
    got = gs.depthwise_conv2d(x.to(DEV), w.to(DEV), (1, 1), (0, 0))
    assert (got.cpu() == 128 * 128 * 9).all()
    # an infinity next to the border must not leak into windows that do not contain it
    xf = torch.zeros((1, 1, 8, 8), dtype=torch.bfloat16)
    xf[0, 0, 0, 7] = float("inf")
    wf = torch.ones((1, 3, 3), dtype=torch.bfloat16)
    gf = gs.depthwise_conv2d(xf.to(DEV), wf.to(DEV), (1, 1), (1, 1)).cpu()
    assert torch.isinf(gf[0, 0, :2, 6:]).all() and torch.isfinite(gf[0, 0, 2:]).all() and torch.isfinite(gf[0, 0, :, :6]).all()
    empty = torch.zeros((0, 4, 8, 8), dtype=torch.bfloat16, device=DEV)
    assert gs.depthwise_conv2d(empty, torch.ones((4, 3, 3), dtype=torch.bfloat16, device=DEV), (1, 1), (1, 1)).shape == (0, 4, 8, 8)


# ---------------------------------------------------------------------------------------------
# seeded random sweeps of the window kernels
# ---------------------------------------------------------------------------------------------

def _random_window_cases(seed, count):
    r = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        dtype = ("i8", "bf16", "f32", "i32")[int(r.integers(4))]
        n, c = int(r.integers(1, 4)), int(r.integers(1, 20))
        h, w = int(r.integers(3, 70)), int(r.integers(3, 70))
        k = (int(r.integers(1, 5)), int(r.integers(1, 5)))
        s = (int(r.integers(1, 4)), int(r.integers(1, 4)))
        p = (int(r.integers(0, k[0])), int(r.integers(0, k[1])))
        if h + 2 * p[0] < k[0] or w + 2 * p[1] < k[1]:
            continue
        cases.append((dtype, (n, c, h, w), k, s, p))
    return cases


@pytest.mark.parametrize("case", _random_window_cases(20210906, 40))
def test_windows_random_shapes(case):
    """Pooling (fused windows + reduceMax / reduceSum) and the explicit gather on seeded random planes,
    windows, strides and paddings; maxima and gathers bit-exact, sums within the accumulation bound."""
    dtype, shape, k, s, p = case
    x = gen(dtype, shape, 3500 + shape[2] + shape[3])
    xd = x.to(DEV)
    xo = to_oracle(x)
    got = gs.windows_reduce(xd, 2, k, s, p, p, gs.GS_MAX)
    np.testing.assert_array_equal(to_oracle(got), pg.max_pool2d(ap.tensor(xo), k, s, p, LOWEST[dtype]).materialize())
    win = gs.access_windows(xd, 2, k, s, p, p, gs.GS_PAD_ZERO)
    want_win = oracle_windows(x, 2, k, s, p, p, 0).materialize()
    np.testing.assert_array_equal(to_oracle(win), want_win)
    odt = {"i8": torch.int32, "i32": torch.int32, "bf16": torch.float32, "f32": torch.float32}[dtype]
    tot = gs.windows_reduce(xd, 2, k, s, p, p, gs.GS_SUM, out_dtype=odt)
    want_sum = want_win.sum(axis=(4, 5))
    if dtype in ("i8", "i32"):
        np.testing.assert_array_equal(to_oracle(tot), want_sum)
    else:
        assert_parity(tot, want_sum, float_tol=1e-4, what=str(case))


def _random_depthwise_cases(seed, count):
    r = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        dtype = ("bf16", "i8")[int(r.integers(2))]
        n, c = int(r.integers(1, 4)), int(r.integers(1, 40))
        h, w = int(r.integers(3, 60)), int(r.integers(3, 60))
        kh, kw = [(3, 3), (3, 3), (5, 5), (1, 1), (2, 3), (4, 2)][int(r.integers(6))]
        s = (int(r.integers(1, 3)), int(r.integers(1, 3)))
        p = (int(r.integers(0, kh)), int(r.integers(0, kw)))
        if h + 2 * p[0] < kh or w + 2 * p[1] < kw:
            continue
        odt = torch.int32 if dtype == "i8" else (torch.bfloat16, torch.float32)[int(r.integers(2))]
        cases.append((dtype, n, c, h, w, kh, kw, s, p, odt, bool(r.integers(2))))
    return cases


@pytest.mark.parametrize("case", _random_depthwise_cases(20210907, 30))
def test_depthwise_random_shapes(case):
    dtype, n, c, h, w_, kh, kw, stride, pad, odt, relu = case
    x = gen(dtype, (n, c, h, w_), 3600 + c + h)
    w = gen(dtype, (c, kh, kw), 3700 + c + kh, 1.0 / np.sqrt(kh * kw) if dtype == "bf16" else 1.0)
    got = gs.depthwise_conv2d(x.to(DEV), w.to(DEV), stride, pad, gs.GS_ACT_RELU if relu else gs.GS_ACT_NONE, odt)
    want = oracle_depthwise(x, w, stride, pad)
    assert_parity(got, np.maximum(want, 0) if relu else want, what=str(case))
