"""Pins of the chained oracle (oracle.network.run) and of the layer table that both the oracle chain and
the packed network read (workloads.resnet18_layers).  No GPU.

The paper names its residual network (Sec. 5.1, Sec. 6.2) but prints no layer list; the table asserted
here is the standard 18-layer residual topology at batch 8.  Every node of a small network of the same
structure is rebuilt from a table written out in this file, by direct calls to the pinned per-layer oracle
functions and, where a library routine computes the same thing (max pooling, the fully connected product,
the integer convolution), by that routine in float64 -- so a wrong source node, a swapped residual, a
transposed fully connected operand or a dropped pooling node in the chain fails here.
"""
import numpy as np
import torch
import torch.nn.functional as F

import oracle
from oracle import network as onet
from paper_2106_12169_amd import workloads as wl

U, P = wl.ENC_UNSIGNED, wl.ENC_PM1

# (name, kind, source, residual source, Cin, Cout, H = W of the input, kernel, stride, pad, q, q_out)
# of the small network: image 32 x 32, widths 32 / 32 / 64 / 64, 10 classes.
SMALL = [
    ("conv1",      "conv",    "image",      None,         3, 32, 32, 7, 2, 3, 8, 2),
    ("maxpool",    "maxpool", "conv1",      None,        32, 32, 16, 3, 2, 1, 2, 2),
    ("s1b1_conv1", "conv",    "maxpool",    None,        32, 32,  8, 3, 1, 1, 2, 2),
    ("s1b1_conv2", "conv",    "s1b1_conv1", "maxpool",   32, 32,  8, 3, 1, 1, 2, 2),
    ("s1b2_conv1", "conv",    "s1b1_conv2", None,        32, 32,  8, 3, 1, 1, 2, 2),
    ("s1b2_conv2", "conv",    "s1b2_conv1", "s1b1_conv2", 32, 32, 8, 3, 1, 1, 2, 2),
    ("s2b1_conv1", "conv",    "s1b2_conv2", None,        32, 32,  8, 3, 2, 1, 2, 2),
    ("s2b1_short", "conv",    "s1b2_conv2", None,        32, 32,  8, 1, 2, 0, 2, 2),
    ("s2b1_conv2", "conv",    "s2b1_conv1", "s2b1_short", 32, 32, 4, 3, 1, 1, 2, 2),
    ("s2b2_conv1", "conv",    "s2b1_conv2", None,        32, 32,  4, 3, 1, 1, 2, 2),
    ("s2b2_conv2", "conv",    "s2b2_conv1", "s2b1_conv2", 32, 32, 4, 3, 1, 1, 2, 2),
    ("s3b1_conv1", "conv",    "s2b2_conv2", None,        32, 64,  4, 3, 2, 1, 2, 2),
    ("s3b1_short", "conv",    "s2b2_conv2", None,        32, 64,  4, 1, 2, 0, 2, 2),
    ("s3b1_conv2", "conv",    "s3b1_conv1", "s3b1_short", 64, 64, 2, 3, 1, 1, 2, 2),
    ("s3b2_conv1", "conv",    "s3b1_conv2", None,        64, 64,  2, 3, 1, 1, 2, 2),
    ("s3b2_conv2", "conv",    "s3b2_conv1", "s3b1_conv2", 64, 64, 2, 3, 1, 1, 2, 2),
    ("s4b1_conv1", "conv",    "s3b2_conv2", None,        64, 64,  2, 3, 2, 1, 2, 2),
    ("s4b1_short", "conv",    "s3b2_conv2", None,        64, 64,  2, 1, 2, 0, 2, 2),
    ("s4b1_conv2", "conv",    "s4b1_conv1", "s4b1_short", 64, 64, 1, 3, 1, 1, 2, 2),
    ("s4b2_conv1", "conv",    "s4b1_conv2", None,        64, 64,  1, 3, 1, 1, 2, 2),
    ("s4b2_conv2", "conv",    "s4b2_conv1", "s4b1_conv2", 64, 64, 1, 3, 1, 1, 2, 2),
    ("sumpool",    "sumpool", "s4b2_conv2", None,        64, 64,  1, 1, 1, 0, 2, 8),
    ("fc",         "fc",      "sumpool",    None,        64, 10,  1, 1, 1, 0, 8, 0),
]
RES_SCALE = 0.5


def _conv_f64(w, x, stride, pad):
    """Integer convolution by the library routine in float64 (exact: every magnitude is far below 2^53)."""
    return F.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                    stride=stride, padding=pad).numpy()


def test_every_node_of_the_small_network_from_a_table_written_here():
    layers = wl.resnet18_layers(image_hw=32, num_classes=10, widths=(32, 32, 64, 64))
    params = wl.network_params(layers)
    img = wl.image_batch(77, 2, 32)
    got = onet.run(layers, params, img)
    assert [L.name for L in layers] == [row[0] for row in SMALL]
    mine = {"image": img}
    for (name, kind, src, res, Cin, Cout, hw, k, stride, pad, q, q_out) in SMALL:
        x = mine[src]
        assert x.shape[1] == Cin and (kind == "fc" or x.shape[2] == hw), name
        if kind == "conv":
            w, sc, bi = params[name]
            assert w.shape == (Cout, Cin, k, k) and set(np.unique(w)) <= {-1, 1}
            acc = oracle.conv2d(w, P, 1, x, U, q, stride, pad)
            assert np.array_equal(acc, _conv_f64(w, x, stride, pad)), name       # library routine, float64
            codes, _ = oracle.epilogue(acc, sc, bi, q_out, res=mine[res] if res else None, res_scale=RES_SCALE)
            # the epilogue away from its rounding boundaries, in double
            td = (np.float64(sc)[None, :, None, None] * acc + np.float64(bi)[None, :, None, None]
                  + (RES_SCALE * mine[res] if res else 0.0))
            safe = np.abs(td - np.round(td)) > 1e-3
            assert safe.mean() > 0.95 and td.shape == codes.shape
            assert np.array_equal(codes[safe], np.clip(np.floor(td), 0, 3).astype(np.uint8)[safe]), name
            mine[name] = codes
        elif kind == "maxpool":
            ref = F.max_pool2d(torch.from_numpy(x.astype(np.float32)), k, stride, pad).numpy().astype(np.uint8)
            assert np.array_equal(oracle.maxpool(x, k, stride, pad), ref)
            mine[name] = ref
        elif kind == "sumpool":
            s = x.astype(np.int64).sum((2, 3))
            assert s.max() < 256
            mine[name] = s.astype(np.uint8)
        else:                                                                     # fc: logits[b][c] = sum_k x[b][k] w[c][k]
            w, _, _ = params[name]
            w2 = w.reshape(Cout, Cin)
            logits = x.astype(np.float64) @ w2.astype(np.float64).T
            assert logits.shape == (2, Cout)
            mine[name] = logits.astype(np.int32)
        assert got[name].shape == mine[name].shape and got[name].dtype == mine[name].dtype, name
        assert np.array_equal(got[name], mine[name]), name
    assert set(got) == set(mine)
    # orientation: a non-square fully connected product differs from its transpose-confused variants
    assert got["fc"].shape == (2, 10) and len(np.unique(got["fc"])) > 5


def test_residual_sources_matter():
    """Swapping in any other node of the same shape as the residual changes the block output."""
    layers = wl.resnet18_layers(image_hw=32, num_classes=10, widths=(32, 32, 64, 64))
    params = wl.network_params(layers)
    got = onet.run(layers, params, wl.image_batch(78, 2, 32))
    L = next(l for l in layers if l.name == "s2b1_conv2")
    w, sc, bi = params[L.name]
    acc = oracle.conv2d(w, P, 1, got["s2b1_conv1"], U, 2, 1, 1)
    right, _ = oracle.epilogue(acc, sc, bi, 2, res=got["s2b1_short"], res_scale=0.5)
    wrong, _ = oracle.epilogue(acc, sc, bi, 2, res=got["s2b1_conv1"], res_scale=0.5)
    assert np.array_equal(right, got[L.name]) and not np.array_equal(wrong, got[L.name])


# The 18-layer residual topology at batch 8, image 224 x 224, 1000 classes:
# (name, kind, source, residual, Cin, Cout, input H = W, kernel, stride, pad, K = Cin R S, output pixels x batch 8)
FULL = [
    ("conv1",      "conv",    "image",      None,          3,  64, 224, 7, 2, 3,  147, 100352),
    ("maxpool",    "maxpool", "conv1",      None,         64,  64, 112, 3, 2, 1, None,  25088),
    ("s1b1_conv1", "conv",    "maxpool",    None,         64,  64,  56, 3, 1, 1,  576,  25088),
    ("s1b1_conv2", "conv",    "s1b1_conv1", "maxpool",    64,  64,  56, 3, 1, 1,  576,  25088),
    ("s1b2_conv1", "conv",    "s1b1_conv2", None,         64,  64,  56, 3, 1, 1,  576,  25088),
    ("s1b2_conv2", "conv",    "s1b2_conv1", "s1b1_conv2", 64,  64,  56, 3, 1, 1,  576,  25088),
    ("s2b1_conv1", "conv",    "s1b2_conv2", None,         64, 128,  56, 3, 2, 1,  576,   6272),
    ("s2b1_short", "conv",    "s1b2_conv2", None,         64, 128,  56, 1, 2, 0,   64,   6272),
    ("s2b1_conv2", "conv",    "s2b1_conv1", "s2b1_short", 128, 128, 28, 3, 1, 1, 1152,   6272),
    ("s2b2_conv1", "conv",    "s2b1_conv2", None,        128, 128,  28, 3, 1, 1, 1152,   6272),
    ("s2b2_conv2", "conv",    "s2b2_conv1", "s2b1_conv2", 128, 128, 28, 3, 1, 1, 1152,   6272),
    ("s3b1_conv1", "conv",    "s2b2_conv2", None,        128, 256,  28, 3, 2, 1, 1152,   1568),
    ("s3b1_short", "conv",    "s2b2_conv2", None,        128, 256,  28, 1, 2, 0,  128,   1568),
    ("s3b1_conv2", "conv",    "s3b1_conv1", "s3b1_short", 256, 256, 14, 3, 1, 1, 2304,   1568),
    ("s3b2_conv1", "conv",    "s3b1_conv2", None,        256, 256,  14, 3, 1, 1, 2304,   1568),
    ("s3b2_conv2", "conv",    "s3b2_conv1", "s3b1_conv2", 256, 256, 14, 3, 1, 1, 2304,   1568),
    ("s4b1_conv1", "conv",    "s3b2_conv2", None,        256, 512,  14, 3, 2, 1, 2304,    392),
    ("s4b1_short", "conv",    "s3b2_conv2", None,        256, 512,  14, 1, 2, 0,  256,    392),
    ("s4b1_conv2", "conv",    "s4b1_conv1", "s4b1_short", 512, 512,  7, 3, 1, 1, 4608,    392),
    ("s4b2_conv1", "conv",    "s4b1_conv2", None,        512, 512,   7, 3, 1, 1, 4608,    392),
    ("s4b2_conv2", "conv",    "s4b2_conv1", "s4b1_conv2", 512, 512,  7, 3, 1, 1, 4608,    392),
    ("sumpool",    "sumpool", "s4b2_conv2", None,        512, 512,   7, 7, 1, 0, None,      8),
    ("fc",         "fc",      "sumpool",    None,        512, 1000,  1, 1, 1, 0,  512,      8),
]


def test_full_size_layer_table():
    layers = wl.resnet18_layers()
    assert len(layers) == len(FULL)
    macs = 0
    for L, (name, kind, src, res, Cin, Cout, hw, k, stride, pad, K, pixels) in zip(layers, FULL):
        assert (L.name, L.kind, L.src, L.res) == (name, kind, src, res), name
        assert (L.Cin, L.Cout, L.H, L.W, L.R, L.S, L.stride, L.pad) == (Cin, Cout, hw, hw, k, k, stride, pad), name
        assert 8 * L.Ho * L.Wo == pixels, name
        if kind in ("conv", "fc"):
            assert L.Cin * L.R * L.S == K, name
            assert L.p == 1
            macs += pixels * Cout * K
        # bit widths: 8-bit image and 8-bit pooled sums, 2-bit codes everywhere else; int32 logits at the end
        assert L.q == (8 if name in ("conv1", "fc") else 2), name
        assert L.q_out == (0 if name == "fc" else 8 if name == "sumpool" else 2), name
        if res:
            assert L.res_scale == 0.5
    # by hand: conv1 944 111 616; stage 1 4 x 924 844 032; stages 2-4 each 462 422 016 + 51 380 224 + 3 x 924 844 032;
    # fc 4 096 000  ->  1.451e10 multiply-accumulates at batch 8
    assert macs == 944_111_616 + 4 * 924_844_032 + 3 * (462_422_016 + 51_380_224 + 3 * 924_844_032) + 4_096_000
    assert macs == 14_512_586_752
    # a block's second convolution reads the first, and adds either the block input or its shortcut convolution
    by = {L.name: L for L in layers}
    for s in range(1, 5):
        for b in (1, 2):
            c1, c2 = by[f"s{s}b{b}_conv1"], by[f"s{s}b{b}_conv2"]
            assert c2.src == c1.name
            short = by.get(f"s{s}b{b}_short")
            assert c2.res == (short.name if short else c1.src)
            if short:
                assert short.src == c1.src and (short.Ho, short.Wo, short.Cout) == (c1.Ho, c1.Wo, c1.Cout)
    # 49 codes of at most 3 fit the 8-bit sum
    assert by["sumpool"].H * by["sumpool"].W * 3 < 256


def test_plain_chains_pooled_nodes_and_full_frame_layers():
    """The chains without shortcuts: a convolution with fused 2 x 2 max pooling is the library's pooling of the
    float64 convolution followed by the epilogue; the first fully connected layer is the product of the flattened
    (channel, row, column) feature map with the flattened weights; shapes as written here."""
    layers = wl.vgg16_layers(image_hw=32, num_classes=10, widths=(32, 32, 64, 64, 64), fc_width=96)
    assert [L.name for L in layers if L.kind == "conv" and L.pool] == ["conv2", "conv4", "conv7", "conv10", "conv13"]
    assert [(L.name, L.H) for L in layers if L.name in ("conv3", "conv5", "conv8", "conv11", "fc6")] == \
        [("conv3", 16), ("conv5", 8), ("conv8", 4), ("conv11", 2), ("fc6", 1)]
    params = wl.network_params(layers)
    img = wl.image_batch(79, 2, 32)
    got = onet.run(layers, params, img)
    by = {L.name: L for L in layers}
    for name in ("conv2", "conv7"):
        L = by[name]
        w, sc, bi = params[name]
        acc = F.max_pool2d(torch.from_numpy(_conv_f64(w, got[L.src], 1, 1)), 2, 2).numpy().astype(np.int32)
        codes, _ = oracle.epilogue(acc, sc, bi, 2)
        assert np.array_equal(codes, got[name]) and codes.shape[2] == L.Ho // 2
    a = wl.alexnet_layers(image_hw=99, num_classes=10, widths=(32, 64, 96, 64, 64), fc_width=128)
    assert [(L.name, L.kind, L.H, L.R, L.stride) for L in a[:4]] == \
        [("conv1", "conv", 99, 11, 4), ("pool1", "maxpool", 24, 3, 2), ("conv2", "conv", 11, 5, 1), ("pool2", "maxpool", 11, 3, 2)]
    pa = wl.network_params(a)
    ga = onet.run(a, pa, wl.image_batch(80, 2, 99))
    L = next(l for l in a if l.name == "fc6")
    assert (L.H, L.R, L.pad, L.Ho) == (2, 2, 0, 1)
    w, sc, bi = pa["fc6"]
    x = ga[L.src].astype(np.float64).reshape(2, -1)                        # (channel, row, column) order
    acc = (x @ w.astype(np.float64).reshape(w.shape[0], -1).T).astype(np.int32).reshape(2, -1, 1, 1)
    codes, _ = oracle.epilogue(acc, sc, bi, 2)
    assert np.array_equal(codes, ga["fc6"])
    # full-size tables: multiply-accumulates per image of the two shapes
    macs = lambda Ls: sum(L.Ho * L.Wo * L.Cout * L.Cin * L.R * L.S for L in Ls if L.kind in ("conv", "fc"))
    assert macs(wl.alexnet_layers()) == 714_188_480 and macs(wl.vgg16_layers()) == 15_470_264_320
