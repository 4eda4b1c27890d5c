"""Seeded synthetic inputs and workload shapes.

Only data is produced here: uniform integers, fair signs, normals and the
shape tables of the benchmark workloads.  None of the method's arithmetic
(bit-plane splitting, packing, AND/XOR+popcount products, shift-add,
epilogue) lives in this module, so the CPU oracle tests and the HIP path can
both draw their inputs from it without sharing any computation.

The generator is counter based: element ``i`` of stream ``seed`` is a pure
function of ``(seed, i)`` (the published splitmix64 output function applied to
``seed * 2^32 + i`` style counters), so any slice of a tensor can be produced
without producing the rest.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

ENC_UNSIGNED = 0  # stored bit b counts as b
ENC_PM1 = 1       # stored bit b counts as 2b-1 (1-bit only)

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def raw_u64(seed: int, start: int, count: int) -> np.ndarray:
    """64 random bits for counters start .. start+count-1 of stream ``seed``."""
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + count, dtype=np.uint64)
        z = (idx + np.uint64(1)) * _GOLDEN + np.uint64(seed) * _M2
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform_codes(seed: int, shape, bits: int) -> np.ndarray:
    """Unsigned integers uniform in [0, 2^bits), one per byte (uint8)."""
    n = int(np.prod(shape))
    r = raw_u64(seed, 0, n) >> np.uint64(64 - bits)
    return r.astype(np.uint8).reshape(shape)


def fair_signs(seed: int, shape) -> np.ndarray:
    """Independent fair -1/+1 values, one per byte (int8)."""
    n = int(np.prod(shape))
    b = (raw_u64(seed, 0, n) >> np.uint64(63)).astype(np.int8)
    return (2 * b - 1).astype(np.int8).reshape(shape)


def normals(seed: int, shape, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """Normal deviates (Box-Muller on two counter streams, in double), as fp32."""
    n = int(np.prod(shape))
    u1 = ((raw_u64(seed, 0, n) >> np.uint64(11)).astype(np.float64) + 1.0) / 9007199254740993.0
    u2 = (raw_u64(seed ^ 0x5DEECE66D, 0, n) >> np.uint64(11)).astype(np.float64) / 9007199254740992.0
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    return (mean + std * z).astype(np.float32).reshape(shape)


def uniform_floats(seed: int, shape, lo: float, hi: float) -> np.ndarray:
    n = int(np.prod(shape))
    u = (raw_u64(seed, 0, n) >> np.uint64(11)).astype(np.float64) / 9007199254740992.0
    return (lo + (hi - lo) * u).astype(np.float32).reshape(shape)


def operand(seed: int, rows: int, K: int, bits: int, enc: int) -> np.ndarray:
    """A rows x K operand in its unpacked one-value-per-byte form."""
    if enc == ENC_PM1:
        assert bits == 1
        return fair_signs(seed, (rows, K))
    return uniform_codes(seed, (rows, K), bits)


# --------------------------------------------------------------------------
# GEMM workloads (benchmark configurations 0, 1, 2)
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class GemmWorkload:
    name: str
    M: int
    N: int
    K: int
    p: int          # weight bits
    q: int          # activation bits
    encW: int
    encX: int
    seedW: int
    seedX: int

    def weights(self) -> np.ndarray:
        return operand(self.seedW, self.M, self.K, self.p, self.encW)

    def activations(self) -> np.ndarray:
        return operand(self.seedX, self.N, self.K, self.q, self.encX)

    @property
    def effective_ops(self) -> float:
        return 2.0 * self.M * self.N * self.K


def gemm_w1a2(n: int, cfg: int) -> GemmWorkload:
    return GemmWorkload(f"gemm_w1a2_{n}", n, n, n, 1, 2, ENC_PM1, ENC_UNSIGNED, 1000 + cfg, 2000 + cfg)


CONFIG0 = gemm_w1a2(128, 0)
CONFIG1 = gemm_w1a2(4096, 1)
SWEEP_BITS: Tuple[Tuple[int, int], ...] = ((1, 1), (1, 2), (2, 2), (1, 4), (3, 5), (2, 8))


def sweep_workload(w: int, a: int, n: int = 2048) -> GemmWorkload:
    return GemmWorkload(f"gemm_w{w}a{a}_{n}", n, n, n, w, a, ENC_UNSIGNED, ENC_UNSIGNED,
                        1002 + 16 * w + a, 2002 + 16 * w + a)


CONFIG2 = tuple(sweep_workload(w, a) for (w, a) in SWEEP_BITS)

# Fully-connected layer shapes of the APMM evaluation (Sec. 6.1.1): batch 64, input = output
# dimension in {128, 256, ..., 1024}; the raw-latency table uses 64 x 1024 x 1024.  Weights are
# the M rows (output neurons), the batch supplies the N rows.  Bit combinations: those named in
# that section and its latency table (unsigned x unsigned, as in the precision sweep).
PAPER_FC_DIMS: Tuple[int, ...] = tuple(range(128, 1025, 128))
PAPER_FC_BITS: Tuple[Tuple[int, int], ...] = ((1, 2), (1, 3), (1, 4), (2, 2))


def paper_fc_workload(w: int, a: int, dim: int, batch: int = 64) -> GemmWorkload:
    return GemmWorkload(f"fc_w{w}a{a}_{batch}x{dim}x{dim}", dim, batch, dim, w, a, ENC_UNSIGNED, ENC_UNSIGNED,
                        5000 + 16 * w + a + dim, 6000 + 16 * w + a + dim)


# --------------------------------------------------------------------------
# Convolution workload (benchmark configuration 3)
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class ConvWorkload:
    name: str
    BS: int
    Cin: int
    H: int
    W: int
    Cout: int
    R: int
    S: int
    stride: int
    pad: int
    p: int
    q: int
    encW: int
    encX: int
    q_out: int
    seed: int

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    def features_nchw(self) -> np.ndarray:
        """Activations in the paper's logical order BS x Cin x H x W."""
        return operand(2000 + self.seed, self.BS * self.Cin, self.H * self.W, self.q,
                       self.encX).reshape(self.BS, self.Cin, self.H, self.W)

    def weights_oihw(self) -> np.ndarray:
        """Weights in the paper's logical order Cout x Cin x R x S."""
        return operand(1000 + self.seed, self.Cout, self.Cin * self.R * self.S, self.p,
                       self.encW).reshape(self.Cout, self.Cin, self.R, self.S)

    def scale(self) -> np.ndarray:
        return normals(3000 + self.seed, (self.Cout,), 0.0, 1.0)

    def bias(self) -> np.ndarray:
        return normals(4000 + self.seed, (self.Cout,), 0.0, 0.1)

    @property
    def effective_ops(self) -> float:
        return 2.0 * self.BS * self.Ho * self.Wo * self.Cout * self.Cin * self.R * self.S


def paper_conv_workload(channels: int, w: int = 1, a: int = 2) -> "ConvWorkload":
    """Convolution shape of the APConv evaluation (Sec. 6.1.2): 16 x 16 feature map, 3 x 3 filter,
    stride 1, batch 1, input = output channels in {128, ..., 1024}; fused 2-bit output."""
    return ConvWorkload(f"conv_w{w}a{a}_1x{channels}x16x16", 1, channels, 16, 16, channels, 3, 3, 1, 1, w, a,
                        ENC_UNSIGNED if w > 1 else ENC_PM1, ENC_UNSIGNED, 2, 7000 + channels + 16 * w + a)


PAPER_CONV_CHANNELS: Tuple[int, ...] = (128, 256, 512, 1024)

CONFIG3 = ConvWorkload("conv_w1a2_8x128x28x28", 8, 128, 28, 28, 128, 3, 3, 1, 1, 1, 2,
                       ENC_PM1, ENC_UNSIGNED, 2, 3)


# --------------------------------------------------------------------------
# ResNet-18-shaped network (benchmark configuration 4)
# --------------------------------------------------------------------------

@dataclass
class NetLayer:
    """One node of the layer chain.  ``src``/``res`` name earlier nodes."""
    name: str
    kind: str                 # "conv" | "maxpool" | "sumpool" | "fc"
    src: str
    Cin: int
    Cout: int
    H: int                    # input height/width
    W: int
    R: int = 1
    S: int = 1
    stride: int = 1
    pad: int = 0
    p: int = 1                # weight bits (always +-1 here)
    q: int = 2                # input activation bits
    q_out: int = 2            # 0 -> int32 output, no requantisation
    res: Optional[str] = None # residual source node (packed q_res-bit codes)
    res_scale: float = 0.0
    pool: int = 0             # conv only: 1 = 2 x 2 max pooling of the int32 results before the epilogue (Sec. 5.2)

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1


def resnet18_layers(image_hw: int = 224, num_classes: int = 1000,
                    widths: Tuple[int, int, int, int] = (64, 128, 256, 512)) -> List[NetLayer]:
    """The standard 18-layer residual topology as a flat list of nodes.

    conv1 7x7/2 (8-bit image planes, +-1 weights) -> maxpool 3x3/2 on 2-bit
    codes -> four stages of two basic blocks (3x3 convs; a stride-2 first conv
    plus a 1x1 stride-2 shortcut conv from stage 2 on) -> global sum pool ->
    fully connected layer on 8-bit sums.  ``image_hw`` and ``widths`` can be
    shrunk for small test networks of the same structure.
    """
    L: List[NetLayer] = []
    hw = image_hw
    L.append(NetLayer("conv1", "conv", "image", 3, widths[0], hw, hw, 7, 7, 2, 3, p=1, q=8, q_out=2))
    hw = L[-1].Ho
    L.append(NetLayer("maxpool", "maxpool", "conv1", widths[0], widths[0], hw, hw, 3, 3, 2, 1, q=2, q_out=2))
    hw = L[-1].Ho
    prev, cin = "maxpool", widths[0]
    for si, cout in enumerate(widths):
        for bi in range(2):
            stride = 2 if (si > 0 and bi == 0) else 1
            tag = f"s{si + 1}b{bi + 1}"
            a = NetLayer(tag + "_conv1", "conv", prev, cin, cout, hw, hw, 3, 3, stride, 1)
            L.append(a)
            if stride == 2 or cin != cout:
                sc = NetLayer(tag + "_short", "conv", prev, cin, cout, hw, hw, 1, 1, stride, 0)
                L.append(sc)
                res = sc.name
            else:
                res = prev
            hw2 = a.Ho
            b = NetLayer(tag + "_conv2", "conv", a.name, cout, cout, hw2, hw2, 3, 3, 1, 1,
                         res=res, res_scale=0.5)
            L.append(b)
            prev, cin, hw = b.name, cout, hw2
    L.append(NetLayer("sumpool", "sumpool", prev, cin, cin, hw, hw, hw, hw, 1, 0, q=2, q_out=8))
    L.append(NetLayer("fc", "fc", "sumpool", cin, num_classes, 1, 1, 1, 1, 1, 0, p=1, q=8, q_out=0))
    return L


def _plain_chain(image_hw: int, num_classes: int, first, body, fc_width: int) -> List[NetLayer]:
    """A chain without shortcuts: an input convolution (Cout, kernel, stride, pad), then `body` items that are either
    ("conv", Cout, kernel, pad, pooled) or ("maxpool", kernel, stride), then three fully connected layers.  The first
    fully connected layer reads the whole last feature map: a convolution whose kernel covers the frame; the second
    is a 1 x 1 convolution on the 1 x 1 map; the third produces int32 logits."""
    L: List[NetLayer] = []
    cout, k, stride, pad = first
    L.append(NetLayer("conv1", "conv", "image", 3, cout, image_hw, image_hw, k, k, stride, pad, p=1, q=8, q_out=2))
    prev, cin, hw = "conv1", cout, L[-1].Ho
    n = 1
    for item in body:
        if item[0] == "conv":
            _, cout, k, pad, pooled = item
            n += 1
            layer = NetLayer(f"conv{n}", "conv", prev, cin, cout, hw, hw, k, k, 1, pad, pool=1 if pooled else 0)
            L.append(layer)
            prev, cin, hw = layer.name, cout, (layer.Ho // 2 if pooled else layer.Ho)
        else:
            _, k, stride = item
            layer = NetLayer(f"pool{n}", "maxpool", prev, cin, cin, hw, hw, k, k, stride, 0, q=2, q_out=2)
            L.append(layer)
            prev, hw = layer.name, layer.Ho
    L.append(NetLayer("fc6", "conv", prev, cin, fc_width, hw, hw, hw, hw, 1, 0))
    L.append(NetLayer("fc7", "conv", "fc6", fc_width, fc_width, 1, 1, 1, 1, 1, 0))
    L.append(NetLayer("fc8", "fc", "fc7", fc_width, num_classes, 1, 1, 1, 1, 1, 0, p=1, q=2, q_out=0))
    return L


def alexnet_layers(image_hw: int = 224, num_classes: int = 1000,
                   widths: Tuple[int, int, int, int, int] = (64, 192, 384, 256, 256), fc_width: int = 4096) -> List[NetLayer]:
    """AlexNet-shaped chain (the paper evaluates an AlexNet variant, Sec. 6.2, without printing its layers; these are
    the widely used single-tower shapes): 11 x 11 / 4 input convolution on the 8-bit image, 3 x 3 / 2 max pooling on
    codes after the first, second and fifth convolution, a 5 x 5 and three 3 x 3 convolutions (1-bit weights, 2-bit
    activations), three fully connected layers."""
    w = widths
    body = [("maxpool", 3, 2), ("conv", w[1], 5, 2, False), ("maxpool", 3, 2), ("conv", w[2], 3, 1, False),
            ("conv", w[3], 3, 1, False), ("conv", w[4], 3, 1, False), ("maxpool", 3, 2)]
    return _plain_chain(image_hw, num_classes, (w[0], 11, 4, 2), body, fc_width)


def vgg16_layers(image_hw: int = 224, num_classes: int = 1000,
                 widths: Tuple[int, int, int, int, int] = (64, 128, 256, 512, 512), fc_width: int = 4096) -> List[NetLayer]:
    """VGG-16-shaped chain (the paper's VGG variant is not printed either): thirteen 3 x 3 convolutions in five groups
    of 2, 2, 3, 3, 3, the last of each group with 2 x 2 max pooling fused into its epilogue (the fusion of Sec. 5.2),
    three fully connected layers."""
    body = []
    for g, (cout, reps) in enumerate(zip(widths, (2, 2, 3, 3, 3))):
        for r in range(reps):
            if g == 0 and r == 0:
                continue                                   # the input convolution
            body.append(("conv", cout, 3, 1, r == reps - 1))
    return _plain_chain(image_hw, num_classes, (widths[0], 3, 1, 1), body, fc_width)


# Assumed (mean, variance) of one input value by the kind of node that produced
# it; used only to place the synthetic folded-BN parameters so that every layer
# keeps using all of its code levels.
_CODE_STATS = (1.5, 1.0)           # floor(N(2, 1)) clamped to {0..3}
_POOLED_STATS = (1.41, 0.5)        # 3x3/2 max of floor(N(0.5, 1)) clamped codes
_IMAGE_STATS = (127.5, (256.0 ** 2 - 1.0) / 12.0)
_FIRST_CENTRE = 0.5                # conv1 sits lower so that max pooling does not saturate


def network_params(layers: List[NetLayer], seed: int = 0):
    """Seeded +-1 weights and folded per-channel a', b' for every conv / fc node.

    Returns {name: (weights Cout x Cin x R x S int8, scale fp32[Cout], bias fp32[Cout])}.
    The synthetic batch-norm statistics are the closed-form ones of a sum of K
    terms w_k x_k with fixed signs w and independent inputs of mean mu and
    variance v:  mean_c = mu * sum_k w[c][k],  var_c = K * v.  The folded scale
    is (1 + 10 % jitter) / sqrt(var_c) and the folded bias centres the pre-floor
    value on 2.0 (0.5 for the first layer) plus N(0, 0.1) jitter, less the mean
    contribution of a residual input.
    """
    kind = {L.name: ("maxpool" if L.kind == "conv" and L.pool else L.kind) for L in layers}
    by_name = {L.name: L for L in layers}
    out = {}
    for i, L in enumerate(layers):
        if L.kind not in ("conv", "fc"):
            continue
        K = L.Cin * L.R * L.S
        w = fair_signs(10_000 + 100 * seed + i, (L.Cout, L.Cin, L.R, L.S))
        src_kind = kind.get(L.src, "image")
        if src_kind == "image":
            mu, v = _IMAGE_STATS
        elif src_kind == "maxpool":
            mu, v = _POOLED_STATS
        elif src_kind == "sumpool":
            hw = by_name[L.src].H * by_name[L.src].W
            mu, v = hw * _CODE_STATS[0], hw * _CODE_STATS[1]
        else:
            mu, v = _CODE_STATS
        wsum = w.astype(np.float64).sum(axis=(1, 2, 3))
        jitter = 1.0 + 0.1 * normals(20_000 + 100 * seed + i, (L.Cout,)).astype(np.float64)
        a = jitter / math.sqrt(K * v)
        # (a layer whose codes go through max pooling sits lower, so that the maximum does not saturate)
        nxt = [M for M in layers if M.src == L.name]
        feeds_pool = L.pool or any(M.kind == "maxpool" for M in nxt)
        centre = _FIRST_CENTRE if (src_kind == "image" or feeds_pool) else 2.0
        if L.res:
            centre -= L.res_scale * _CODE_STATS[0]
        b = centre - a * mu * wsum + normals(30_000 + 100 * seed + i, (L.Cout,), 0.0, 0.1).astype(np.float64)
        out[L.name] = (w, a.astype(np.float32), b.astype(np.float32))
    return out


def image_batch(seed: int, batch: int, hw: int) -> np.ndarray:
    """Uniform 8-bit image batch in the usual batch x 3 x H x W order."""
    return uniform_codes(seed, (batch, 3, hw, hw), 8)
