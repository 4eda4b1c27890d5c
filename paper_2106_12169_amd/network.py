"""Layer chaining for a packed-activation network (minimal-traffic dataflow,
Sec. 5.1): marshalling only.

Weights are packed once at construction (off the timed path, as in Sec. 5.1);
``forward`` enqueues one library call per node on the current stream: the 8-bit
image goes to the input layer as it is, every other convolution reads packed
bit planes and writes packed bit planes through the fused epilogue, the last
layer produces int32 logits without requantisation.  All buffers are
preallocated so that ``forward`` can be captured in a HIP graph.
"""

from __future__ import annotations

from typing import Dict, List

import numpy as np
import torch

from . import binding as B
from .workloads import NetLayer


class PackedNet:
    def __init__(self, layers: List[NetLayer], params: Dict[str, tuple], batch: int, device="cuda", fuse_tail: bool = True):
        """fuse_tail: a global sum pooling whose only reader is the last fully connected layer shares that layer's
        launch (apnn_sumpool_fc); its own buffer is then not written."""
        self.layers, self.batch, self.dev = layers, batch, device
        self.fused_tail = None
        if (fuse_tail and len(layers) >= 2 and layers[-1].kind == "fc" and layers[-2].kind == "sumpool"
                and layers[-1].src == layers[-2].name and layers[-2].q_out == 8 and layers[-2].Cin <= 4096
                and not any(L.src == layers[-2].name or L.res == layers[-2].name for L in layers[:-1])):
            self.fused_tail = layers[-2].name
        self.w, self.scale, self.bias, self.buf = {}, {}, {}, {}
        self.geom = {}
        self._by_name = {L.name: L for L in layers}
        first = layers[0]
        for L in layers:
            if L.kind in ("conv", "fc"):
                wv, sc, bi = params[L.name]
                wd = torch.from_numpy(np.ascontiguousarray(wv)).to(device)
                if L is first:
                    self.w[L.name] = B.apnn_pack_input_weights(wd, L.p, B.ENC_PM1)
                elif L.kind == "fc" and self._by_name[L.src].kind == "sumpool":
                    self.w[L.name] = B.apnn_pack(wd.reshape(L.Cout, -1), L.p, B.ENC_PM1)       # matrix operand
                else:
                    self.w[L.name] = B.apnn_pack_conv_weights(wd, L.p, B.ENC_PM1)
                self.scale[L.name] = torch.from_numpy(sc).to(device)
                self.bias[L.name] = torch.from_numpy(bi).to(device)
            pixels = batch * (L.Ho // 2) * (L.Wo // 2) if (L.kind == "conv" and L.pool) else batch * L.Ho * L.Wo
            if L.kind == "fc":
                self.buf[L.name] = torch.empty((batch, L.Cout), dtype=torch.int32, device=device)
            elif L.kind == "sumpool":
                self.buf[L.name] = torch.empty(B.apnn_packed_words(batch, L.Cout, L.q_out), dtype=torch.int32, device=device)
            else:
                self.buf[L.name] = torch.empty(B.apnn_fmap_words(pixels, L.Cout, L.q_out), dtype=torch.int32, device=device)
        torch.cuda.synchronize()

    def _conv_args(self, L: NetLayer) -> dict:
        d = B.Conv(self.batch, L.H, L.W, L.Cin, L.Cout, L.R, L.S, L.stride, L.pad, L.p, L.q)
        return dict(d=d, W=self.w[L.name], X=self.buf[L.src], q_out=L.q_out, scale=self.scale[L.name],
                    bias=self.bias[L.name], residual=self.buf[L.res] if L.res else None,
                    q_res=self._by_name[L.res].q_out if L.res else 0,
                    res_scale=L.res_scale, out=self.buf[L.name], pool=B.POOL_MAX2 if L.pool else B.POOL_NONE)

    def forward(self, image: torch.Tensor) -> torch.Tensor:
        """image: batch x 3 x H x W uint8 device tensor -> int32 logits batch x classes."""
        first = self.layers[0]
        paired = None
        self.launches = 0                               # library calls (= kernel launches) of this pass
        for i, L in enumerate(self.layers):
            out = self.buf[L.name]
            if L is paired:
                continue
            self.launches += 1
            if L is first:
                d = B.Conv(self.batch, L.H, L.W, L.Cin, L.Cout, L.R, L.S, L.stride, L.pad, L.p, L.q)
                B.apnn_input_layer(d, self.w[L.name], image, q_out=L.q_out,
                                   scale=self.scale[L.name], bias=self.bias[L.name], out=out)
            elif L.kind == "conv":
                nxt = self.layers[i + 1] if i + 1 < len(self.layers) else None
                if (nxt is not None and nxt.kind == "conv" and nxt.src == L.src
                        and nxt.res != L.name and L.res != nxt.name and not L.pool and not nxt.pool):
                    # two convolutions of the same features that do not depend on each other (a down-sampling
                    # block's 3 x 3 convolution and its 1 x 1 shortcut): one call, one launch
                    B.apnn_layer_pair(self._conv_args(L), self._conv_args(nxt))
                    paired = nxt
                else:
                    a = self._conv_args(L)
                    B.apnn_layer(a.pop("d"), a.pop("W"), a.pop("X"), **a)
            elif L.kind == "maxpool":
                B.apnn_maxpool(self.buf[L.src], self.batch, L.H, L.W, L.Cin, L.q, L.R, L.stride, L.pad, out=out)
            elif L.kind == "sumpool":
                if L.name == self.fused_tail:
                    self.launches -= 1                  # computed in the launch of the layer that reads it
                    continue
                B.apnn_sumpool(self.buf[L.src], self.batch, L.H, L.W, L.Cin, L.q, L.q_out, out=out)
            elif L.kind == "fc" and L.src == self.fused_tail:
                S = self._by_name[L.src]
                B.apnn_sumpool_fc(self.buf[S.src], self.batch, S.H, S.W, S.Cin, S.q, self.w[L.name], L.Cout, L.p,
                                  B.ENC_PM1, out=out)
            elif L.kind == "fc":
                # the pooled sums are a matrix operand; a 1 x 1 feature map is read as one (a 1 x 1 convolution)
                d = B.Conv(self.batch, 1, 1, L.Cin, L.Cout, 1, 1, 1, 0, L.p, L.q)
                B.apnn_layer(d, self.w[L.name], self.buf[L.src], is_gemm=self._by_name[L.src].kind == "sumpool", acc_out=out)
            else:
                raise ValueError(L.kind)
        return self.buf[self.layers[-1].name]
