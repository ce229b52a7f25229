"""GPU parity at the sizes of the five workloads.  Where the oracle cannot evaluate a whole
workload in seconds it evaluates whole images of it: every operator here treats the batch
dimension as an access dimension, so image n of the GPU result must equal the oracle's result on
image n alone."""

import numpy as np
import pytest
import torch

from oracle import access_pattern as ap, brute, programs as pg, resnet as oresnet
from paper_2105_09377_amd import binding as gs, synth
from paper_2105_09377_amd.resnet import ResNet18Stack
from helpers import assert_parity, to_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ODT = {"i8": torch.int32, "bf16": torch.bfloat16}


def _conv_images(cfg, images, form, odt, residual=None, act=gs.GS_ACT_NONE):
    x, w = cfg["x"], cfg["w"]
    fn = gs.conv2d_direct if form == "direct" else gs.conv2d_im2col
    got = fn(x.to(DEV), w.to(DEV), cfg["stride"], cfg["pad"], out_dtype=odt, act=act,
             residual=None if residual is None else residual.to(DEV))
    idx = torch.tensor(images)
    want = brute.conv2d(to_oracle(x[idx]), to_oracle(w), cfg["stride"], cfg["pad"])
    if residual is not None:
        want = want + to_oracle(residual[idx])
    if act == gs.GS_ACT_RELU:
        want = np.maximum(want, 0)
    return got, got[idx.to(DEV)], want


def test_config1_tiny_conv_three_ways():
    cfg = synth.tiny_conv_int8()
    x, w = cfg["x"], cfg["w"]
    want = brute.conv2d(to_oracle(x), to_oracle(w), (1, 1), (0, 0))
    prog = pg.conv2d(ap.tensor(to_oracle(x)), ap.tensor(to_oracle(w)), (1, 1)).materialize()
    np.testing.assert_array_equal(prog, want)
    a = gs.conv2d_direct(x.to(DEV), w.to(DEV))
    b = gs.conv2d_im2col(x.to(DEV), w.to(DEV))
    assert_parity(a, want)
    assert torch.equal(a, b)


def test_config2_mlp():
    cfg = synth.mlp_bf16()
    h = cfg["x"].to(DEV)
    ref = to_oracle(cfg["x"])
    for i, w in enumerate(cfg["weights"]):
        last = i == len(cfg["weights"]) - 1
        h = gs.cartesian_dot(h, w.to(DEV), out_dtype=torch.float32 if last else torch.bfloat16,
                             act=gs.GS_ACT_NONE if last else gs.GS_ACT_RELU)
        ref = brute.matmul(ref, to_oracle(w).T)
        if not last:
            from oracle import numerics
            ref = numerics.round_to_bf16_value(np.maximum(ref, 0))
        assert_parity(h, ref, what=f"layer {i}")


@pytest.mark.parametrize("form", ["direct", "im2col"])
@pytest.mark.parametrize("dtype", ["bf16", "i8"])
def test_config3_resnet_conv3x3(dtype, form):
    cfg = synth.resnet_conv3x3(dtype, 32)
    _, got, want = _conv_images(cfg, [0, 13, 31], form, ODT[dtype])
    assert_parity(got, want, what=f"{dtype} {form}")


def test_config4_downsample_block():
    blk = synth.downsample_block(32)
    x = blk["x"]
    images = [0, 17, 31]
    main = {"x": x, "w": blk["w3"], "stride": (2, 2), "pad": (1, 1)}
    proj = {"x": x, "w": blk["w1"], "stride": (2, 2), "pad": (0, 0)}
    p_full, p_got, p_want = _conv_images(proj, images, "direct", torch.bfloat16)
    assert_parity(p_got, p_want, what="projection")
    # main path + projection (reduceSum over the pair) + ReLU.  The oracle adds the projection
    # exactly as the GPU stored it (bfloat16), so both sides add the same values and the sum is
    # held to the same bound as every other layer.
    from oracle import numerics
    idx = torch.tensor(images)
    s_full, s_got, _ = _conv_images(main, images, "direct", torch.bfloat16, residual=p_full.cpu(), act=gs.GS_ACT_RELU)
    want = brute.conv2d(to_oracle(x[idx]), to_oracle(blk["w3"]), (2, 2), (1, 1)) + to_oracle(p_full.cpu()[idx])
    want = np.maximum(want, 0)
    assert_parity(s_got, want, what="block sum")
    pooled = gs.windows_reduce(s_full, 2, (2, 2), (2, 2), None, None, gs.GS_MAX)
    assert pooled.shape == (32, 256, 7, 7)
    # pooling is exact: check it on the block output the oracle computed
    want_pool = brute.max_pool2d(numerics.round_to_bf16_value(want), (2, 2), (2, 2), (0, 0), -np.inf)
    dev_in = torch.from_numpy(numerics.round_to_bf16_value(want)).to(torch.bfloat16).to(DEV)
    got_pool = gs.windows_reduce(dev_in, 2, (2, 2), (2, 2), None, None, gs.GS_MAX)
    np.testing.assert_array_equal(to_oracle(got_pool), want_pool)


# -- configuration 5: every distinct layer at batch 64, then the whole stack at a reduced size ----

LAYER_SHAPES = sorted({(cin, cout, k, s, p, hw) for (_n, cin, cout, k, s, p), hw in zip(
    synth.RESNET18_CONVS,
    [224, 56, 56, 56, 56, 56, 28, 56, 28, 28, 28, 14, 28, 14, 14, 14, 7, 14, 7, 7])})


@pytest.mark.parametrize("shape", LAYER_SHAPES)
def test_config5_layer_at_batch_64(shape):
    cin, cout, k, s, p, hw = shape
    cfg = synth.conv_layer(64, cin, hw, hw, cout, k, s, p, "bf16", 7000 + cin + 7 * cout + k + s, gain=2.0 ** 0.5)
    _, got, want = _conv_images(cfg, [0, 40, 63], "direct", torch.bfloat16, act=gs.GS_ACT_RELU)
    assert_parity(got, want, what=str(shape))
    if cin < 16:        # the stem also in the im2col-rewritten form
        _, got2, _ = _conv_images(cfg, [0, 40, 63], "im2col", torch.bfloat16, act=gs.GS_ACT_RELU)
        assert_parity(got2, want, what=str(shape) + " im2col")


def test_config5_pool_avg_fc_at_batch_64():
    x = synth.normal_bf16((64, 64, 112, 112), 1.0, 7101)
    got = gs.windows_reduce(x.to(DEV), 2, (3, 3), (2, 2), (1, 1), (1, 1), gs.GS_MAX)
    idx = torch.tensor([0, 29, 63])
    want = brute.max_pool2d(to_oracle(x[idx]), (3, 3), (2, 2), (1, 1), -np.inf)
    np.testing.assert_array_equal(to_oracle(got[idx.to(DEV)]), want)
    y = synth.normal_bf16((64, 512, 7, 7), 1.0, 7102)
    avg = gs.reduce(y.to(DEV), 2, gs.GS_SUM, scale=1.0 / 49)
    assert_parity(avg, to_oracle(y).reshape(64, 512, 49).sum(axis=2) / 49.0, what="avg")
    a = synth.normal_bf16((64, 512), 1.0, 7103)
    w = synth.normal_bf16((1000, 512), 512 ** -0.5, 7104)
    fc = gs.cartesian_dot(a.to(DEV), w.to(DEV))
    assert_parity(fc, brute.matmul(to_oracle(a), to_oracle(w).T), what="fc")


def _check_stack(net, x, weights, images):
    """One forward pass of the stack against the oracle on whole images.

    Layer by layer ("teacher forced"): each layer's oracle result is computed from the inputs of
    that layer exactly as the GPU stored them (bfloat16 activations, residual included), so every
    stored value is held to the element-wise relative bound.  End to end: the logits against the
    oracle's own forward pass.  Both sides store bfloat16 between layers, and an activation that
    the two accumulation orders round to different bfloat16 values (one ulp) perturbs every output
    of the next layer by a small ABSOLUTE amount, so logits near zero cannot be held to a relative
    bound after twenty layers; the chain is held to 1e-2 of the largest logit.
    """
    from oracle import numerics
    logits = net.forward(x.to(DEV))
    idx = torch.tensor(images)
    w64 = {k: to_oracle(v) for k, v in weights.items()}
    spec = {name: (k, s, p) for name, _ci, _co, k, s, p in synth.RESNET18_CONVS}

    def stored(name):
        return to_oracle(net.bufs[name][idx.to(DEV)])

    def layer(name, src, residual=None, relu=True):
        k, s, p = spec[name]
        want = brute.conv2d(src, w64[name], (s, s), (p, p))
        if residual is not None:
            want = want + residual
        if relu:
            want = np.maximum(want, 0)
        assert_parity(net.bufs[name][idx.to(DEV)], want, what=name)
        return stored(name)

    y = layer("conv1", to_oracle(x[idx]))
    want_pool = brute.max_pool2d(y, (3, 3), (2, 2), (1, 1), -np.inf)
    np.testing.assert_array_equal(stored("pool"), want_pool)          # max is exact
    y = stored("pool")
    for stage in (1, 2, 3, 4):
        for block in (1, 2):
            pre = f"s{stage}b{block}"
            t = layer(pre + "c1", y)
            shortcut = layer(pre + "proj", y, relu=False) if (pre + "proj") in spec else y
            y = layer(pre + "c2", t, residual=shortcut)
    n, c, h, w = y.shape
    assert_parity(net.bufs["avg"][idx.to(DEV)], y.reshape(n, c, h * w).sum(axis=2) / (h * w), what="avg")
    assert_parity(logits[idx.to(DEV)], brute.matmul(stored("avg"), w64["fc"].T), what="fc")
    # end to end
    ref = oresnet.forward(to_oracle(x[idx]), w64, synth.RESNET18_CONVS)
    got = to_oracle(logits[idx.to(DEV)])
    err = np.abs(got - ref["fc"]).max() / np.abs(ref["fc"]).max()
    assert err <= 1e-2, f"logits end to end: max error {err:.3e} of the largest logit"
    return logits


def test_config5_whole_stack_reduced_size():
    cfg = synth.resnet18_stack(batch=2, image=64, classes=100)
    net = ResNet18Stack(cfg["weights"], batch=2, image=64, device=DEV)
    logits = _check_stack(net, cfg["x"], cfg["weights"], [0, 1])
    # same input again through the same buffers: deterministic
    again = net.forward().clone()
    assert torch.equal(again, logits)


def test_config5_whole_stack_full_size():
    """The workload that `bench.py` times: batch 64 at 224x224, every layer buffer and the logits
    (projections in the im2col form, residual + ReLU at 56/28/14/7, the split channel sums of the
    last stage), on whole images."""
    cfg = synth.resnet18_stack(batch=64)
    net = ResNet18Stack(cfg["weights"], batch=64, image=224, device=DEV)
    _check_stack(net, cfg["x"], cfg["weights"], [0, 37, 63])
