"""ResNet-18-shaped convolution stack as a fixed sequence of library calls.

Every layer is one access-pattern program of the paper evaluated by the HIP library:

* 3x3 and 7x7 convolutions are Fig. 2a (`conv2d_direct_packed`, windows formed on chip; the
  3-channel stem takes the library's few-channel kernel, which forms im2col rows in LDS);
* the 1x1 stride-2 shortcut projections have no window overlap to exploit, so they run in the
  im2col-rewritten form of Fig. 5 (`conv2d_im2col`: explicit gather, then the dense contraction),
  which is the faster of the two forms for them;
* ReLU and the residual addition (the `reduceSum (pair a b)` idiom of Sec. 5.4) are fused into the
  convolution epilogues;
* max pooling is Fig. 2c (`windows_reduce`), the global average is `compute reduceSum` with a
  scale (`reduce`), the classifier is `compute dotProd (cartProd ...)` (`cartesian_dot`).

This module only sequences calls and owns the buffers; it does no arithmetic.  No batch-norm and
no biases: the stack exercises the operators the paper defines, with the layer shapes of the network.
"""

from __future__ import annotations

from typing import Callable, Dict, List, Tuple

import torch

from . import binding as gs
from .synth import RESNET18_CONVS


class ResNet18Stack:
    def __init__(self, weights: Dict[str, torch.Tensor], batch: int, image: int, device="cuda:0"):
        self.dev = torch.device(device)
        self.batch, self.image = batch, image
        self.w = {k: v.to(self.dev) for k, v in weights.items()}
        self.spec = {name: (cin, cout, k, s, p) for name, cin, cout, k, s, p in RESNET18_CONVS}
        self.bufs: Dict[str, torch.Tensor] = {}
        self.x = torch.empty((batch, 3, image, image), dtype=torch.bfloat16, device=self.dev)
        h = self._out(image, 7, 2, 3)
        self._alloc("conv1", (batch, 64, h, h))
        h = self._out(h, 3, 2, 1)
        self._alloc("pool", (batch, 64, h, h))
        # Weights are constants: pack them once, in the order the contraction reads them, each
        # into a buffer sized for its layer's call (weights plus that call's scratch).
        self.packed: Dict[str, torch.Tensor] = {}
        self.packed["conv1"] = self._pack("conv1", tuple(self.x.shape), 2, 3)
        ws_bytes = 0
        for name, (cin, cout, k, s, p) in self.spec.items():
            if name == "conv1":
                continue
            if name.endswith("c1"):
                hin = h
                h = self._out(h, k, s, p)
            elif name.endswith("proj"):
                assert self._out(hin, k, s, p) == h
            src_hw = hin if name.endswith(("c1", "proj")) else h
            if name.endswith("proj"):
                ws_bytes = max(ws_bytes, gs.conv2d_workspace(self.x, self.w[name], (s, s), (p, p), form="im2col",
                                                             x_shape=(batch, cin, src_hw, src_hw)))
            else:
                self.packed[name] = self._pack(name, (batch, cin, src_hw, src_hw), s, p)
            self._alloc(name, (batch, cout, h, h))
        self.ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=self.dev)   # shared by the projections
        self._alloc("avg", (batch, 512))
        self.logits = torch.empty((batch, self.w["fc"].shape[0]), dtype=torch.float32, device=self.dev)
        self.steps = self.plan()

    def _pack(self, name: str, x_shape: Tuple[int, ...], s: int, p: int) -> torch.Tensor:
        need = gs.conv2d_workspace(self.x, self.w[name], (s, s), (p, p), x_shape=x_shape)
        buf = torch.empty(max(need, 16), dtype=torch.uint8, device=self.dev)
        return gs.conv2d_pack_weights(self.w[name], packed=buf)

    @staticmethod
    def _out(h: int, k: int, s: int, p: int) -> int:
        return (h + 2 * p - k) // s + 1

    def _alloc(self, name: str, shape: Tuple[int, ...]) -> None:
        self.bufs[name] = torch.empty(shape, dtype=torch.bfloat16, device=self.dev)

    def _conv(self, name: str, x: torch.Tensor, residual=None, relu=True) -> torch.Tensor:
        _cin, _cout, k, s, p = self.spec[name]
        if name.endswith("proj"):
            return gs.conv2d_im2col(x, self.w[name], (s, s), (p, p), residual=residual,
                                    act=gs.GS_ACT_RELU if relu else gs.GS_ACT_NONE, out=self.bufs[name],
                                    workspace=self.ws)
        return gs.conv2d_direct_packed(x, self.w[name], self.packed[name], (s, s), (p, p), residual=residual,
                                       act=gs.GS_ACT_RELU if relu else gs.GS_ACT_NONE, out=self.bufs[name])

    def layer_calls(self) -> List[str]:
        """Names of the library calls of one forward pass, in order."""
        return ["conv1", "pool"] + [n for n in self.spec if n != "conv1"] + ["avg", "fc"]

    def plan(self) -> List[Tuple[str, Callable[[], torch.Tensor]]]:
        """The forward pass as (layer name, call) pairs in execution order.  Every call reads and
        writes this object's fixed buffers, so a call can be launched (and timed) on its own once
        the calls before it have run."""
        b = self.bufs
        steps: List[Tuple[str, Callable[[], torch.Tensor]]] = [
            ("conv1", lambda: self._conv("conv1", self.x)),
            ("pool", lambda: gs.windows_reduce(b["conv1"], 2, (3, 3), (2, 2), (1, 1), (1, 1), gs.GS_MAX, out=b["pool"])),
        ]
        y = "pool"
        for stage in (1, 2, 3, 4):
            for block in (1, 2):
                pre = f"s{stage}b{block}"
                steps.append((pre + "c1", lambda pre=pre, y=y: self._conv(pre + "c1", b[y])))
                shortcut = y
                if (pre + "proj") in self.spec:
                    steps.append((pre + "proj", lambda pre=pre, y=y: self._conv(pre + "proj", b[y], relu=False)))
                    shortcut = pre + "proj"
                steps.append((pre + "c2", lambda pre=pre, sc=shortcut: self._conv(pre + "c2", b[pre + "c1"], residual=b[sc])))
                y = pre + "c2"
        hw = b[y].shape[-1] * b[y].shape[-2]
        steps.append(("avg", lambda y=y: gs.reduce(b[y], 2, gs.GS_SUM, scale=1.0 / hw, out=b["avg"])))
        steps.append(("fc", lambda: gs.cartesian_dot(b["avg"], self.w["fc"], out=self.logits)))
        return steps

    def forward(self, x: torch.Tensor = None) -> torch.Tensor:
        if x is not None:
            self.x.copy_(x)
        out = None
        for _name, call in self.steps:
            out = call()
        return out
