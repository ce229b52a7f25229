"""Pins for the stack oracle (oracle/resnet.py): it must agree with an independent library
evaluation of the same network (torch CPU float64 convolution / pooling / linear routines with
torch's own bfloat16 rounding between layers) and keep the structural facts of the network."""

import numpy as np
import torch
import torch.nn.functional as F

from oracle import resnet as oresnet
from paper_2105_09377_amd import synth
from helpers import to_oracle


def _library_forward(x, w, convs):
    spec = {name: (k, s, p) for name, _ci, _co, k, s, p in convs}
    rb = lambda t: t.to(torch.bfloat16).to(torch.float64)

    def conv(name, a, residual=None, relu=True):
        k, s, p = spec[name]
        y = F.conv2d(a, w[name], stride=s, padding=p)
        if residual is not None:
            y = y + residual
        return rb(F.relu(y) if relu else y)

    inter = {}
    y = inter["conv1"] = conv("conv1", x)
    y = inter["pool"] = F.max_pool2d(y, 3, 2, 1)
    for stage in (1, 2, 3, 4):
        for block in (1, 2):
            pre = f"s{stage}b{block}"
            t = conv(pre + "c1", y)
            sc = conv(pre + "proj", y, relu=False) if (pre + "proj") in spec else y
            y = inter[pre + "c2"] = conv(pre + "c2", t, residual=sc)
    avg = rb(y.mean(dim=(2, 3)))
    inter["fc"] = avg @ w["fc"].t()
    return inter


def test_stack_oracle_matches_library_routines():
    cfg = synth.resnet18_stack(batch=1, image=32, classes=24)
    x = to_oracle(cfg["x"])
    w = {k: to_oracle(v) for k, v in cfg["weights"].items()}
    got = oresnet.forward(x, w, synth.RESNET18_CONVS)
    ref = _library_forward(torch.from_numpy(x), {k: torch.from_numpy(v) for k, v in w.items()},
                           synth.RESNET18_CONVS)
    assert got["fc"].shape == (1, 24)
    for name in ("conv1", "pool", "s1b2c2", "s2b1c2", "s3b2c2", "s4b2c2", "fc"):
        g, r = got[name], ref[name].numpy()
        assert g.shape == r.shape, name
        # Both sides round to bfloat16 after every layer; a sum that lands within an fp64 rounding
        # of a tie may round differently (one bfloat16 ulp = 2^-8 relative) and feed the next layers.
        scale = np.abs(r).max()
        assert np.abs(g - r).max() <= 2.0 ** -7 * scale, name
        assert (g != r).mean() < 0.02, name


def test_stack_oracle_structure():
    cfg = synth.resnet18_stack(batch=1, image=32, classes=8)
    w = {k: to_oracle(v) for k, v in cfg["weights"].items()}
    zero = oresnet.forward(np.zeros((1, 3, 32, 32)), w, synth.RESNET18_CONVS)
    assert all(np.all(v == 0) for v in zero.values())          # no biases anywhere
    out = oresnet.forward(to_oracle(cfg["x"]), w, synth.RESNET18_CONVS)
    assert out["conv1"].shape == (1, 64, 16, 16) and out["pool"].shape == (1, 64, 8, 8)
    assert out["s2b1c1"].shape == (1, 128, 4, 4) and out["s4b2c2"].shape == (1, 512, 1, 1)
    for name, v in out.items():
        if name.endswith(("c1", "c2")) or name in ("conv1", "pool", "avg"):
            assert v.min() >= 0, name                          # ReLU outputs and their pool / mean
    assert out["s2b1proj"].min() < 0                           # the projection has no ReLU
    # a block whose second convolution has zero weights passes its shortcut through unchanged
    w2 = dict(w)
    w2["s1b1c2"] = np.zeros_like(w["s1b1c2"])
    out2 = oresnet.forward(to_oracle(cfg["x"]), w2, synth.RESNET18_CONVS)
    np.testing.assert_array_equal(out2["s1b1c2"], out2["pool"])
