"""Seeded synthetic inputs for the access-pattern workloads.

The paper evaluates on no dataset and prints no tensors; the workloads are CNN
and MLP layer *shapes*, so random tensors of those shapes stand in.  This
module only draws numbers: it holds none of the method's arithmetic and is the
one piece of code that both the GPU tests and the CPU oracle's tests use, so
that both sides see the same bytes.

Generator: numpy's PCG64 seeded with `BASE_SEED + stream`.  Real-valued tensors
are drawn in float32 and stored as bfloat16 (torch's round-to-nearest-even
cast); integer tensors are drawn uniformly from an inclusive range.
"""

from __future__ import annotations

import math
from typing import Dict, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 210509377


def _rng(stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + int(stream)))


def normal_bf16(shape: Sequence[int], scale: float, stream: int) -> torch.Tensor:
    """N(0,1) * scale, stored as a CPU bfloat16 tensor."""
    x = _rng(stream).standard_normal(tuple(shape), dtype=np.float32) * np.float32(scale)
    return torch.from_numpy(x).to(torch.bfloat16)


def normal_fp8(shape: Sequence[int], scale: float, stream: int) -> torch.Tensor:
    """N(0,1) * scale, stored as a CPU float8_e4m3fn tensor (torch's round-to-nearest-even cast;
    values beyond +-448 would become NaN in that cast, so they are clipped first)."""
    x = _rng(stream).standard_normal(tuple(shape), dtype=np.float32) * np.float32(scale)
    return torch.from_numpy(np.clip(x, -448.0, 448.0)).to(torch.float8_e4m3fn)


def uniform_int8(shape: Sequence[int], lo: int, hi: int, stream: int) -> torch.Tensor:
    """Integers uniform in [lo, hi] inclusive, stored as a CPU int8 tensor."""
    x = _rng(stream).integers(lo, hi + 1, size=tuple(shape), dtype=np.int64)
    return torch.from_numpy(x.astype(np.int8))


def uniform_int32(shape: Sequence[int], lo: int, hi: int, stream: int) -> torch.Tensor:
    x = _rng(stream).integers(lo, hi + 1, size=tuple(shape), dtype=np.int64)
    return torch.from_numpy(x.astype(np.int32))


def normal_f32(shape: Sequence[int], scale: float, stream: int) -> torch.Tensor:
    x = _rng(stream).standard_normal(tuple(shape), dtype=np.float32) * np.float32(scale)
    return torch.from_numpy(x)


# ---------------------------------------------------------------------------
# The five workloads
# ---------------------------------------------------------------------------

def tiny_conv_int8() -> Dict[str, object]:
    """1x3x8x8 input, 4x3x3x3 weights, stride 1, no padding, integers in [-8, 8]."""
    return {"x": uniform_int8((1, 3, 8, 8), -8, 8, 101),
            "w": uniform_int8((4, 3, 3, 3), -8, 8, 102),
            "stride": (1, 1), "pad": (0, 0)}


def mlp_bf16(batch: int = 256, dims: Sequence[int] = (784, 512, 512, 10)) -> Dict[str, object]:
    """Dense layers; weights stored [out, in] and scaled by 1/sqrt(fan_in)."""
    ws = [normal_bf16((dims[i + 1], dims[i]), 1.0 / math.sqrt(dims[i]), 210 + i)
          for i in range(len(dims) - 1)]
    return {"x": normal_bf16((batch, dims[0]), 1.0, 201), "weights": ws}


def conv_layer(n: int, c: int, h: int, w: int, o: int, k: int, stride: int, pad: int,
               dtype: str, stream: int, gain: float = 1.0) -> Dict[str, object]:
    """One conv layer's activations and weights (weights scaled by gain/sqrt(fan_in))."""
    if dtype == "bf16":
        x = normal_bf16((n, c, h, w), 1.0, stream)
        wt = normal_bf16((o, c, k, k), gain / math.sqrt(c * k * k), stream + 1)
    elif dtype == "i8":
        x = uniform_int8((n, c, h, w), -127, 127, stream)
        wt = uniform_int8((o, c, k, k), -127, 127, stream + 1)
    else:
        raise ValueError(dtype)
    return {"x": x, "w": wt, "stride": (stride, stride), "pad": (pad, pad)}


def resnet_conv3x3(dtype: str = "bf16", n: int = 32) -> Dict[str, object]:
    """N x 64 x 56 x 56 -> 64 channels, 3x3, stride 1, pad 1."""
    return conv_layer(n, 64, 56, 56, 64, 3, 1, 1, dtype, 301 if dtype == "bf16" else 311)


def downsample_block(n: int = 32) -> Dict[str, object]:
    """N x 128 x 28 x 28: 3x3/2 pad 1 -> 256 channels, plus the 1x1/2 projection."""
    main = conv_layer(n, 128, 28, 28, 256, 3, 2, 1, "bf16", 401)
    proj_w = normal_bf16((256, 128, 1, 1), 1.0 / math.sqrt(128), 405)
    return {"x": main["x"], "w3": main["w"], "w1": proj_w}


#: (name, C_in, C_out, kernel, stride, pad) of every convolution of the ResNet-18-shaped stack,
#: in execution order; "proj" layers are the 1x1 shortcuts of the downsampling blocks.
RESNET18_CONVS: Tuple[Tuple[str, int, int, int, int, int], ...] = (
    ("conv1", 3, 64, 7, 2, 3),
    ("s1b1c1", 64, 64, 3, 1, 1), ("s1b1c2", 64, 64, 3, 1, 1),
    ("s1b2c1", 64, 64, 3, 1, 1), ("s1b2c2", 64, 64, 3, 1, 1),
    ("s2b1c1", 64, 128, 3, 2, 1), ("s2b1c2", 128, 128, 3, 1, 1), ("s2b1proj", 64, 128, 1, 2, 0),
    ("s2b2c1", 128, 128, 3, 1, 1), ("s2b2c2", 128, 128, 3, 1, 1),
    ("s3b1c1", 128, 256, 3, 2, 1), ("s3b1c2", 256, 256, 3, 1, 1), ("s3b1proj", 128, 256, 1, 2, 0),
    ("s3b2c1", 256, 256, 3, 1, 1), ("s3b2c2", 256, 256, 3, 1, 1),
    ("s4b1c1", 256, 512, 3, 2, 1), ("s4b1c2", 512, 512, 3, 1, 1), ("s4b1proj", 256, 512, 1, 2, 0),
    ("s4b2c1", 512, 512, 3, 1, 1), ("s4b2c2", 512, 512, 3, 1, 1),
)


def resnet18_stack(batch: int = 64, image: int = 224, classes: int = 1000) -> Dict[str, object]:
    """Input image batch and every weight of the ResNet-18-shaped stack (no batch-norm, no bias).

    Weights are N(0,1) * sqrt(2 / fan_in) so activations stay O(1) through the
    ReLU layers.
    """
    weights = {}
    for i, (name, cin, cout, k, _s, _p) in enumerate(RESNET18_CONVS):
        weights[name] = normal_bf16((cout, cin, k, k), math.sqrt(2.0 / (cin * k * k)), 510 + i)
    weights["fc"] = normal_bf16((classes, 512), math.sqrt(1.0 / 512), 590)
    return {"x": normal_bf16((batch, 3, image, image), 1.0, 501), "weights": weights}
