"""TEST INFRASTRUCTURE ONLY -- CPU oracle of the ResNet-18-shaped stack.

The stack is a composition of the paper's programs: 2D convolution (Fig. 2a), max pooling
(Fig. 2c), element-wise addition as reduceSum over a pair (Sec. 5.4), reduceSum (Table 2) and the
dense layer (Fig. 2b).  Each layer is evaluated by the plain nested loops of `brute.c` in fp64;
between layers the activations are rounded to bfloat16, the storage type the workload fixes for
them (logits stay unrounded).  ReLU and the 1/(H*W) scale of the average are extensions the
workload adds to the paper's operators.
"""

from __future__ import annotations

from typing import Dict, Sequence, Tuple

import numpy as np

from . import brute, numerics


def _r(a: np.ndarray) -> np.ndarray:
    return numerics.round_to_bf16_value(a)


def forward(x: np.ndarray, weights: Dict[str, np.ndarray],
            convs: Sequence[Tuple[str, int, int, int, int, int]]) -> Dict[str, np.ndarray]:
    """x (N,3,H,W) and weights as float64 arrays holding bfloat16 values; `convs` lists
    (name, C_in, C_out, kernel, stride, pad).  Returns every intermediate, keyed like the layers."""
    spec = {name: (k, s, p) for name, _ci, _co, k, s, p in convs}
    out: Dict[str, np.ndarray] = {}

    def conv(name, a, residual=None, relu=True):
        k, s, p = spec[name]
        y = brute.conv2d(a, weights[name], (s, s), (p, p))
        if residual is not None:
            y = y + residual
        if relu:
            y = np.maximum(y, 0.0)
        out[name] = _r(y)
        return out[name]

    y = conv("conv1", x)
    y = out["pool"] = brute.max_pool2d(y, (3, 3), (2, 2), (1, 1), -np.inf)
    for stage in (1, 2, 3, 4):
        for block in (1, 2):
            pre = f"s{stage}b{block}"
            t = conv(pre + "c1", y)
            shortcut = conv(pre + "proj", y, relu=False) if (pre + "proj") in spec else y
            y = conv(pre + "c2", t, residual=shortcut)
    n, c, h, w = y.shape
    avg = out["avg"] = _r(y.reshape(n, c, h * w).sum(axis=2) * (1.0 / (h * w)))
    out["fc"] = brute.matmul(avg, weights["fc"].T)     # dense layer: weights stored [out, in]
    return out
