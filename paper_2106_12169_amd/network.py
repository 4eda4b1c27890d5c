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
    def __init__(self, layers: List[NetLayer], params: Dict[str, tuple], batch: int, device="cuda"):
        self.layers, self.batch, self.dev = layers, batch, device
        self.w, self.scale, self.bias, self.buf = {}, {}, {}, {}
        self.geom = {}
        first = layers[0]
        for L in layers:
            if L.kind in ("conv", "fc"):
                wv, sc, bi = params[L.name]
                wd = torch.from_numpy(np.ascontiguousarray(wv)).to(device)
                if L is first:
                    self.w[L.name] = B.apnn_pack_input_weights(wd, L.p, B.ENC_PM1)
                elif L.kind == "fc":
                    self.w[L.name] = B.apnn_pack(wd.reshape(L.Cout, -1), L.p, B.ENC_PM1)
                else:
                    self.w[L.name] = B.apnn_pack_conv_weights(wd, L.p, B.ENC_PM1)
                self.scale[L.name] = torch.from_numpy(sc).to(device)
                self.bias[L.name] = torch.from_numpy(bi).to(device)
            pixels = batch * L.Ho * L.Wo
            if L.kind == "fc":
                self.buf[L.name] = torch.empty((batch, L.Cout), dtype=torch.int32, device=device)
            elif L.kind == "sumpool":
                self.buf[L.name] = torch.empty(B.apnn_packed_words(batch, L.Cout, L.q_out), dtype=torch.int32, device=device)
            else:
                self.buf[L.name] = torch.empty(B.apnn_fmap_words(pixels, L.Cout, L.q_out), dtype=torch.int32, device=device)
        torch.cuda.synchronize()

    def forward(self, image: torch.Tensor) -> torch.Tensor:
        """image: batch x 3 x H x W uint8 device tensor -> int32 logits batch x classes."""
        first = self.layers[0]
        for L in self.layers:
            out = self.buf[L.name]
            if L is first:
                d = B.Conv(self.batch, L.H, L.W, L.Cin, L.Cout, L.R, L.S, L.stride, L.pad, L.p, L.q)
                B.apnn_input_layer(d, self.w[L.name], image, q_out=L.q_out,
                                   scale=self.scale[L.name], bias=self.bias[L.name], out=out)
            elif L.kind == "conv":
                d = B.Conv(self.batch, L.H, L.W, L.Cin, L.Cout, L.R, L.S, L.stride, L.pad, L.p, L.q)
                B.apnn_layer(d, self.w[L.name], self.buf[L.src], q_out=L.q_out,
                             scale=self.scale[L.name], bias=self.bias[L.name],
                             residual=self.buf[L.res] if L.res else None, q_res=2, res_scale=L.res_scale, out=out)
            elif L.kind == "maxpool":
                B.apnn_maxpool(self.buf[L.src], self.batch, L.H, L.W, L.Cin, L.q, L.R, L.stride, L.pad, out=out)
            elif L.kind == "sumpool":
                B.apnn_sumpool(self.buf[L.src], self.batch, L.H, L.W, L.Cin, L.q, L.q_out, out=out)
            elif L.kind == "fc":
                d = B.Conv(self.batch, 1, 1, L.Cin, L.Cout, 1, 1, 1, 0, L.p, L.q)
                B.apnn_layer(d, self.w[L.name], self.buf[L.src], is_gemm=True, acc_out=out)
            else:
                raise ValueError(L.kind)
        return self.buf[self.layers[-1].name]
