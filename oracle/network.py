"""Oracle for a chain of layers (test infrastructure only).

Walks a list of layer nodes (conv / maxpool / sumpool / fc) and applies the
plain oracle functions in the paper's logical tensor orders: integer
convolution, then the fused scale/bias(+residual) -> floor -> clamp step
(Sec. 5.1 dataflow, Sec. 5.2 fused form).  The paper gives no layer list for
its residual network, so the wiring used here (identity or 1x1-conv shortcut
codes added inside the second conv's epilogue, max pooling on codes, global
sum pooling, a final fully connected layer with int32 logits and no
requantisation) is this build's reading.  Pinned node by node (source and
residual nodes, pooling, operand orientation of the last layer) against a
layer table written out in tests/test_oracle_network_pins.py.
"""

from __future__ import annotations

import numpy as np

from . import POOL_MAX, conv2d, epilogue, gemm, gridpool, maxpool, sumpool

ENC_UNSIGNED, ENC_PM1 = 0, 1


def run(layers, params, image_nchw):
    """params[name] = (weights Cout x Cin x R x S int8 +-1, scale, bias).

    Returns {node name: uint8 codes (BS x C x H x W) or int32 logits (BS x C)}.
    """
    out = {"image": np.ascontiguousarray(image_nchw, np.uint8)}
    for L in layers:
        x = out[L.src]
        if L.kind == "conv":
            w, scale, bias = params[L.name]
            acc = conv2d(w, ENC_PM1, L.p, x, ENC_UNSIGNED, L.q, L.stride, L.pad)
            if getattr(L, "pool", 0):                   # 2 x 2 max pooling of the integer results, then the epilogue (Sec. 5.2)
                acc = gridpool(acc, 2, POOL_MAX)
            res = out[L.res] if L.res else None
            codes, _ = epilogue(acc, scale, bias, L.q_out, res=res, res_scale=L.res_scale)
            out[L.name] = codes
        elif L.kind == "maxpool":
            out[L.name] = maxpool(x, L.R, L.stride, L.pad)
        elif L.kind == "sumpool":
            out[L.name] = sumpool(x)
        elif L.kind == "fc":
            w, scale, bias = params[L.name]
            # logits[b][c] = sum_k X[b][k] * W[c][k]: activations are the row operand
            out[L.name] = gemm(x.reshape(x.shape[0], -1), ENC_UNSIGNED, L.q,
                               w.reshape(w.shape[0], -1), ENC_PM1, L.p)
        else:
            raise ValueError(L.kind)
    return out
