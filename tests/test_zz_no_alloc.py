"""The entry point that allocates nothing: `glenside_conv2d_direct_static` against
`glenside_conv2d_direct`, through the C ABI, on two calls in a row (the second smaller), sharing
the library's fixed scratch array."""

import ctypes
import gc

import pytest
import torch

from paper_2105_09377_amd import binding as gs, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(cfg, odt, residual=None, act=gs.GS_ACT_NONE):
    x, w = cfg["x"].to(DEV), cfg["w"].to(DEV)
    res = None if residual is None else residual.to(DEV)
    want = gs.conv2d_direct(x, w, cfg["stride"], cfg["pad"], residual=res, act=act, out_dtype=odt)
    out = torch.empty_like(want)
    gc.collect()                                            # tensors of earlier tests go now, not during the call
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = gs.conv2d_direct_static(x, w, cfg["stride"], cfg["pad"], residual=res, act=act, out=out)
    assert torch.cuda.memory_allocated() <= before          # torch allocated nothing for the call
    torch.cuda.synchronize()
    assert got.data_ptr() == out.data_ptr()
    return got, want


def test_static_scratch_matches_workspace_entry_point_twice():
    # first call: 512 channels at 7x7, a four-way split channel sum (packed weights and partial
    # sums both live in the scratch array), fused residual and ReLU
    big = synth.conv_layer(2, 512, 7, 7, 512, 3, 1, 1, "bf16", 9100, gain=2.0 ** 0.5)
    res = synth.normal_bf16((2, 512, 7, 7), 1.0, 9102)
    got, want = _both(big, torch.bfloat16, residual=res, act=gs.GS_ACT_RELU)
    assert torch.equal(got, want)
    assert got.abs().max() > 0
    # second call, smaller, on the scratch the first one left behind: the tiny int8 workload
    # (few-channel kernel, a second weight copy behind the first)
    small = synth.tiny_conv_int8()
    got2, want2 = _both(small, torch.int32)
    assert torch.equal(got2, want2)
    # and a mid-sized one without split
    mid = synth.conv_layer(3, 64, 20, 20, 96, 3, 2, 1, "bf16", 9110)
    got3, want3 = _both(mid, torch.float32)
    assert torch.equal(got3, want3)


def test_static_scratch_limit():
    limit = gs.conv2d_direct_static_limit()
    assert limit == 32 << 20
    x = torch.zeros((1, 2048, 4, 4), dtype=torch.bfloat16, device=DEV)
    w = torch.zeros((2048, 2048, 3, 3), dtype=torch.bfloat16, device=DEV)
    assert gs.conv2d_workspace(x, w, (1, 1), (1, 1)) > limit
    out = torch.full((1, 2048, 4, 4), 7.0, dtype=torch.float32, device=DEV)
    with pytest.raises(gs.GlensideError) as err:
        gs.conv2d_direct_static(x, w, (1, 1), (1, 1), out=out)
    assert err.value.status == gs.GS_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (out == 7.0).all()                               # nothing was launched
