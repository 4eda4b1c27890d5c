"""GPU parity of apnn_conv2d / apnn_layer / pooling against the oracle:
int32 accumulators and requantised codes bit-exact, fp32 pre-floor values
within 1e-5 relative (they are in fact the same single fma)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2106_12169_amd import binding as B
from paper_2106_12169_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu
U, P = wl.ENC_UNSIGNED, wl.ENC_PM1


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.fixture(params=["auto", "pop8", "pop4", "pop2", "mfma32", "mfma32split1", "mfma32split4", "mfma32split1wide2", "mfma32chunked", "mfma64", "mfma128", "mfma256"])
def tile(request):
    """Kernel path under test: the library's own choice, the AND+popcount kernel with
    each register tile, or the FP4 matrix-core kernel with each block tile."""
    B.apnn_debug_reset()
    kind = request.param
    if kind.startswith("mfma32split1wide"):             # one wave tile of 32 x 64 / 32 x 128 outputs per wave
        B.apnn_debug_force("MFMA_TILE", 32)
        B.apnn_debug_force("MFMA_NSPLIT", 1)
        B.apnn_debug_force("MFMA_FN", int(kind[-1]))
    elif kind.startswith("pop"):
        B.apnn_debug_force("MFMA", 0)
        B.apnn_debug_force("TILE", int(kind[3:]))
    elif kind.startswith("mfma32split"):                # lane-private small-layer kernel, forced K split
        B.apnn_debug_force("MFMA_TILE", 32)
        B.apnn_debug_force("MFMA_NSPLIT", int(kind[-1]))
    elif kind == "mfma32chunked":                      # K-split tile with the chunked loop instead of the resident one
        B.apnn_debug_force("MFMA_TILE", 32)
        B.apnn_debug_force("MFMA_SMALL", 0)
    elif kind.startswith("mfma"):
        B.apnn_debug_force("MFMA_TILE", int(kind[4:]))
    return kind


def run_conv(Wv, encW, p, Xv, q, stride, pad):
    Cout, Cin, R, S = Wv.shape
    N, _, H, Wd = Xv.shape
    d = B.Conv(N, H, Wd, Cin, Cout, R, S, stride, pad, p, q, encW, U)
    Wp = B.apnn_pack_conv_weights(dev(Wv), p, encW)
    Xp = B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, q, U)
    Y = B.apnn_conv2d(d, Wp, Xp)
    torch.cuda.synchronize()
    return Y.cpu().numpy().transpose(0, 3, 1, 2), d, Wp, Xp     # -> N x Cout x Ho x Wo


CONVS = [
    # Cin, Cout, H, W, R, stride, pad, encW, p, q, batch
    (128, 128, 28, 28, 3, 1, 1, P, 1, 2, 2),     # configuration-3 family (vector width 4)
    (64, 64, 14, 14, 3, 1, 1, P, 1, 2, 3),       # 2 channel words
    (64, 128, 15, 13, 3, 2, 1, P, 1, 2, 2),      # stride 2, odd frame
    (64, 128, 14, 14, 1, 2, 0, P, 1, 2, 2),      # 1x1 stride-2 shortcut
    (32, 32, 9, 9, 3, 1, 1, P, 1, 2, 1),         # 1 channel word
    (96, 64, 8, 8, 3, 1, 1, U, 2, 3, 1),         # 3 channel words, unsigned weights
    (256, 96, 7, 7, 3, 1, 1, P, 1, 2, 2),        # Cout not a multiple of the tile
    (128, 64, 6, 6, 5, 1, 2, U, 1, 1, 1),        # 5x5
    (512, 512, 7, 7, 3, 1, 1, P, 1, 2, 1),       # last-stage shape
]


@pytest.mark.parametrize("Cin,Cout,H,Wd,R,stride,pad,encW,p,q,BS", CONVS)
def test_conv2d_matches_oracle(tile, Cin, Cout, H, Wd, R, stride, pad, encW, p, q, BS):
    Wv = wl.operand(31 + Cin + Cout, Cout, Cin * R * R, p, encW).reshape(Cout, Cin, R, R)
    Xv = wl.uniform_codes(32 + H, (BS, Cin, H, Wd), q)
    got, *_ = run_conv(Wv, encW, p, Xv, q, stride, pad)
    assert np.array_equal(got, oracle.conv2d(Wv, encW, p, Xv, U, q, stride, pad))


def _force(force):
    """"auto", a matrix-core block tile ("64", "32split1", "32split4", "32split1wide2") or the AND+popcount kernel
    with a register tile ("pop8", "pop4", "pop2")."""
    B.apnn_debug_reset()
    if force.startswith("pop"):
        B.apnn_debug_force("MFMA", 0)
        B.apnn_debug_force("TILE", int(force[3:]))
    elif force != "auto":
        B.apnn_debug_force("MFMA_TILE", int(force[:2]))
        if force.startswith("32split"):
            B.apnn_debug_force("MFMA_NSPLIT", int(force[7]))
        if "wide" in force:                             # 32 x 64 / 32 x 128 wave tiles
            B.apnn_debug_force("MFMA_FN", int(force[-1]))


ALL_FORMS = ["auto", "64", "32split1", "32split4", "32split1wide2", "pop8", "pop4", "pop2"]

PM1_FEATURE_CONVS = [
    # Cin, Cout, H, W, R, stride, pad, encW, p, BS
    (64, 64, 14, 14, 3, 1, 1, P, 1, 2),          # Case II with padding: overhang taps must contribute 0, not -1
    (128, 96, 9, 11, 3, 2, 1, P, 1, 1),          # stride 2, odd frame, Cout not a multiple of the tile
    (64, 32, 8, 8, 1, 1, 0, P, 1, 2),            # 1x1, no padding
    (64, 64, 7, 7, 5, 1, 2, U, 2, 1),            # mirrored Case III: unsigned 2-bit weights, two rings of overhang
    (256, 64, 6, 6, 3, 1, 1, U, 1, 1),
    (64, 64, 56, 56, 3, 1, 1, P, 1, 1),          # enough output pixels for the 64 x 64 block tile
    (32, 64, 10, 9, 3, 1, 1, P, 1, 2),           # one channel word: only the AND+popcount kernel has this shape
    (96, 32, 7, 8, 3, 2, 2, U, 3, 1),            # three channel words, three weight planes, two rings of padding
    (160, 64, 5, 5, 4, 1, 2, P, 1, 1),           # K words not a multiple of the LDS read group
]


@pytest.mark.parametrize("force", ALL_FORMS)
@pytest.mark.parametrize("Cin,Cout,H,Wd,R,stride,pad,encW,p,BS", PM1_FEATURE_CONVS)
def test_conv_with_pm1_features_matches_oracle(force, Cin, Cout, H, Wd, R, stride, pad, encW, p, BS):
    """-1/+1 features (Case II and the mirrored Case III) with zero-contribution padding, in the matrix-core form (the
    overhang taps become FP4 zeros) and in the AND+popcount form (validity plane that counts negatively)."""
    _force(force)
    Wv = wl.operand(41 + Cin + Cout, Cout, Cin * R * R, p, encW).reshape(Cout, Cin, R, R)
    Xv = wl.fair_signs(42 + H, (BS, Cin, H, Wd))
    d = B.Conv(BS, H, Wd, Cin, Cout, R, R, stride, pad, p, 1, encW, P)
    Y = B.apnn_conv2d(d, B.apnn_pack_conv_weights(dev(Wv), p, encW), B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, 1, P))
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy().transpose(0, 3, 1, 2), oracle.conv2d(Wv, encW, p, Xv, P, 1, stride, pad))


def test_binary_network_chain():
    """Two chained w1a1 layers: the first requantises to 1-bit codes, which the second reads as -1/+1."""
    BS, C, H = 2, 64, 12
    W1, W2 = wl.fair_signs(61, (C, C, 3, 3)), wl.fair_signs(62, (C, C, 3, 3))
    Xv = wl.fair_signs(63, (BS, C, H, H))
    scale = (wl.normals(64, (C,), 1.0, 0.2) / np.sqrt(9.0 * C)).astype(np.float32)
    bias = wl.normals(65, (C,), 1.0, 0.3)
    d = B.Conv(BS, H, H, C, C, 3, 3, 1, 1, 1, 1, P, P)
    mid = B.apnn_layer(d, B.apnn_pack_conv_weights(dev(W1), 1, P), B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, 1, P),
                       q_out=1, scale=dev(scale), bias=dev(bias))
    Y = B.apnn_conv2d(d, B.apnn_pack_conv_weights(dev(W2), 1, P), mid)
    torch.cuda.synchronize()
    codes, _ = oracle.epilogue(oracle.conv2d(W1, P, 1, Xv, P, 1, 1, 1), scale, bias, 1)
    assert 0.2 < codes.mean() < 0.8
    want = oracle.conv2d(W2, P, 1, (2 * codes.astype(np.int8) - 1), P, 1, 1, 1)
    assert np.array_equal(Y.cpu().numpy().transpose(0, 3, 1, 2), want)


def test_pm1_feature_layer_with_epilogue_on_the_popcount_kernel():
    """-1/+1 features through the whole fused layer (scale/bias, residual, requantise, repack) on the literal kernel."""
    B.apnn_debug_force("MFMA", 0)
    BS, Cin, Cout, H = 2, 96, 64, 11
    Wv = wl.fair_signs(51, (Cout, Cin, 3, 3))
    Xv = wl.fair_signs(52, (BS, Cin, H, H))
    scale = (wl.normals(53, (Cout,), 1.0, 0.2) / np.sqrt(9.0 * Cin)).astype(np.float32)
    bias = wl.normals(54, (Cout,), 1.5, 0.3)
    res = wl.uniform_codes(55, (BS, Cout, H, H), 2)
    d = B.Conv(BS, H, H, Cin, Cout, 3, 3, 1, 1, 1, 1, P, P)
    acc = torch.empty((BS, H, H, Cout), dtype=torch.int32, device="cuda")
    out = B.apnn_layer(d, B.apnn_pack_conv_weights(dev(Wv), 1, P), B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, 1, P),
                       q_out=2, scale=dev(scale), bias=dev(bias), acc_out=acc,
                       residual=B.apnn_pack_fmap(dev(res), B.LAYOUT_NCHW, 2, U), q_res=2, res_scale=0.5)
    torch.cuda.synchronize()
    want_acc = oracle.conv2d(Wv, P, 1, Xv, P, 1, 1, 1)
    want_codes, _ = oracle.epilogue(want_acc, scale, bias, 2, res=res, res_scale=0.5)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), want_acc)
    codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), BS, H, H, Cout, 2)
    assert np.array_equal(codes, want_codes) and pad_bits == 0
    assert len(np.unique(want_codes)) == 4


def _layer_case(BS, Cin, Cout, H, R, stride, pad, q, q_out, with_res, seed):
    Wv = wl.fair_signs(seed, (Cout, Cin, R, R))
    Xv = wl.uniform_codes(seed + 1, (BS, Cin, H, H), q)
    K = Cin * R * R
    scale = (wl.normals(seed + 2, (Cout,), 1.0, 0.2) / np.sqrt(K * 3.5)).astype(np.float32)
    bias = wl.normals(seed + 3, (Cout,), 0.5 * (1 << q_out), 0.3)
    d = B.Conv(BS, H, H, Cin, Cout, R, R, stride, pad, 1, q, P, U)
    res = wl.uniform_codes(seed + 4, (BS, Cout, d.Ho, d.Wo), 2) if with_res else None
    return Wv, Xv, scale, bias, res, d


@pytest.mark.parametrize("BS,Cin,Cout,H,R,stride,pad,q,q_out,with_res", [
    (2, 128, 128, 14, 3, 1, 1, 2, 2, False),
    (2, 128, 128, 14, 3, 1, 1, 2, 2, True),
    (1, 64, 64, 12, 3, 1, 1, 2, 2, True),
    (2, 64, 96, 9, 3, 2, 1, 2, 3, False),
    (1, 256, 32, 7, 3, 1, 1, 2, 1, True),
    (1, 64, 160, 8, 1, 1, 0, 2, 8, False),
])
def test_fused_layer_matches_oracle(tile, BS, Cin, Cout, H, R, stride, pad, q, q_out, with_res):
    Wv, Xv, scale, bias, res, d = _layer_case(BS, Cin, Cout, H, R, stride, pad, q, q_out, with_res, 50 + Cin + q_out)
    Wp = B.apnn_pack_conv_weights(dev(Wv), 1, P)
    Xp = B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, q, U)
    resp = B.apnn_pack_fmap(dev(res), B.LAYOUT_NCHW, 2, U) if with_res else None
    acc = torch.empty((d.N, d.Ho, d.Wo, Cout), dtype=torch.int32, device="cuda")
    tf = torch.empty((d.N, d.Ho, d.Wo, Cout), dtype=torch.float32, device="cuda")
    out = B.apnn_layer(d, Wp, Xp, q_out=q_out, scale=dev(scale), bias=dev(bias), residual=resp, q_res=2,
                       res_scale=0.5, acc_out=acc, float_out=tf)
    torch.cuda.synchronize()
    want_acc = oracle.conv2d(Wv, P, 1, Xv, U, q, stride, pad)
    want_codes, want_t = oracle.epilogue(want_acc, scale, bias, q_out, res=res, res_scale=0.5, want_t=True)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), want_acc)
    got_t = tf.cpu().numpy().transpose(0, 3, 1, 2)
    assert np.allclose(got_t, want_t, rtol=1e-5, atol=0) and np.array_equal(got_t, want_t)
    codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), d.N, d.Ho, d.Wo, Cout, q_out)
    assert np.array_equal(codes, want_codes) and pad_bits == 0
    assert len(np.unique(want_codes)) == (1 << q_out) if q_out <= 3 else True


def test_config3_full_layer():
    """Configuration 3 as given (N(0,1) scale, N(0,0.1) bias) and a spread variant
    that exercises all four codes."""
    c = wl.CONFIG3
    Wv, Xv = c.weights_oihw(), c.features_nchw()
    d = B.Conv(c.BS, c.H, c.W, c.Cin, c.Cout, c.R, c.S, c.stride, c.pad, c.p, c.q, c.encW, c.encX)
    Wp = B.apnn_pack_conv_weights(dev(Wv), c.p, c.encW)
    Xp = B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, c.q, c.encX)
    want_acc = oracle.conv2d(Wv, c.encW, c.p, Xv, c.encX, c.q, c.stride, c.pad)
    for scale, bias in ((c.scale(), c.bias()), ((c.scale() / 64).astype(np.float32), (c.bias() + 1.5).astype(np.float32))):
        acc = torch.empty((d.N, d.Ho, d.Wo, c.Cout), dtype=torch.int32, device="cuda")
        tf = torch.empty((d.N, d.Ho, d.Wo, c.Cout), dtype=torch.float32, device="cuda")
        out = B.apnn_layer(d, Wp, Xp, q_out=c.q_out, scale=dev(scale), bias=dev(bias), acc_out=acc, float_out=tf)
        torch.cuda.synchronize()
        want_codes, want_t = oracle.epilogue(want_acc, scale, bias, c.q_out, want_t=True)
        assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), want_acc)
        got_t = tf.cpu().numpy().transpose(0, 3, 1, 2)
        rel = np.abs(got_t - want_t) / np.maximum(np.abs(want_t), 1e-30)
        assert rel.max() <= 1e-5
        codes, _ = hp.unpack_fmap(hp.words_u32(out), d.N, d.Ho, d.Wo, c.Cout, c.q_out)
        assert np.array_equal(codes, want_codes)
    assert len(np.unique(want_codes)) == 4


@pytest.mark.parametrize("channels", wl.PAPER_CONV_CHANNELS)
def test_paper_conv_shapes(channels):
    """Convolution shapes of the paper's APConv evaluation (16 x 16 map, 3 x 3, stride 1, batch 1),
    fused w1a2 layer, default dispatch; the scale is spread so that all four codes occur."""
    c = wl.paper_conv_workload(channels)
    Wv, Xv = c.weights_oihw(), c.features_nchw()
    d = B.Conv(c.BS, c.H, c.W, c.Cin, c.Cout, c.R, c.S, c.stride, c.pad, c.p, c.q, c.encW, c.encX)
    scale = (c.scale() / np.sqrt(9.0 * channels)).astype(np.float32)
    bias = (c.bias() + 1.5).astype(np.float32)
    acc = torch.empty((d.N, d.Ho, d.Wo, c.Cout), dtype=torch.int32, device="cuda")
    out = B.apnn_layer(d, B.apnn_pack_conv_weights(dev(Wv), c.p, c.encW), B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, c.q, c.encX),
                       q_out=c.q_out, scale=dev(scale), bias=dev(bias), acc_out=acc)
    torch.cuda.synchronize()
    want_acc = oracle.conv2d(Wv, c.encW, c.p, Xv, c.encX, c.q, c.stride, c.pad)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), want_acc)
    codes, _ = hp.unpack_fmap(hp.words_u32(out), d.N, d.Ho, d.Wo, c.Cout, c.q_out)
    want_codes, _ = oracle.epilogue(want_acc, scale, bias, c.q_out)
    assert np.array_equal(codes, want_codes) and len(np.unique(want_codes)) == 4


def test_gemm_layer_fc_shape():
    """Fully connected layer: 8-bit activations x +-1 weights, int32 logits, ragged Cout."""
    BS, K, Cout = 8, 512, 1000
    Xv = wl.uniform_codes(1, (BS, K), 8)
    Wv = wl.fair_signs(2, (Cout, K))
    d = B.Conv(BS, 1, 1, K, Cout, 1, 1, 1, 0, 1, 8, P, U)
    logits = torch.empty((BS, Cout), dtype=torch.int32, device="cuda")
    B.apnn_layer(d, B.apnn_pack(dev(Wv), 1, P), B.apnn_pack(dev(Xv), 8, U), is_gemm=True, acc_out=logits)
    torch.cuda.synchronize()
    assert np.array_equal(logits.cpu().numpy(), oracle.gemm(Xv, U, 8, Wv, P, 1))


@pytest.mark.parametrize("k,stride,pad,bits,C,H", [(3, 2, 1, 2, 64, 13), (2, 2, 0, 2, 32, 8), (3, 1, 1, 3, 96, 6),
                                                  (5, 2, 2, 2, 32, 11), (3, 2, 1, 8, 32, 9), (1, 1, 0, 1, 64, 5)])
def test_maxpool(k, stride, pad, bits, C, H):
    Xv = wl.uniform_codes(3, (2, C, H, H), bits)
    Xp = B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, bits, U)
    out = B.apnn_maxpool(Xp, 2, H, H, C, bits, k, stride, pad)
    want = oracle.maxpool(Xv, k, stride, pad)
    codes, _ = hp.unpack_fmap(hp.words_u32(out), 2, want.shape[2], want.shape[3], C, bits)
    assert np.array_equal(codes, want)


@pytest.mark.parametrize("BS,C,H", [(3, 512, 7), (3, 64, 3), (3, 96, 5), (260, 256, 4), (1100, 40, 2), (2100, 130, 2)])
def test_sumpool(BS, C, H):
    """Small batches take the sixteen-wave blocks, large ones a wave per (image, 64 channels)."""
    Xv = wl.uniform_codes(4, (BS, C, H, H), 2)
    Xp = B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, 2, U)
    out = B.apnn_sumpool(Xp, BS, H, H, C, 2, 8)
    codes, pad = hp.unpack_matrix(hp.words_u32(out), BS, C, 8)
    assert np.array_equal(codes, oracle.sumpool(Xv)) and pad == 0


@pytest.mark.parametrize("BS,C,H,Wd,bits,Cout,p,encW", [
    (8, 512, 7, 7, 2, 1000, 1, P),       # the tail of the ResNet-18-shaped network
    (3, 64, 3, 5, 2, 10, 1, P),          # few images, few channel words: many threads share an item's pixels
    (19, 96, 4, 4, 4, 33, 3, U),         # ragged image group and class tile, unsigned 3-bit weights, 4-bit codes
    (1, 32, 1, 1, 8, 1, 8, U),           # one pixel, one word, 8 x 8 bits
    (9, 1024, 2, 2, 1, 70, 2, U),        # 32 words: eight threads each
    (5, 8192, 3, 3, 3, 64, 1, P),        # the most channels allowed: one thread per word
    (300, 64, 2, 3, 2, 1000, 1, P),      # a large batch takes class tiles of 256
])
def test_sumpool_fc(BS, C, H, Wd, bits, Cout, p, encW):
    """Global sum pooling + fully connected layer in one launch against the two oracle steps."""
    Xv = wl.uniform_codes(5 + C, (BS, C, H, Wd), bits)
    Wv = wl.operand(6 + Cout, Cout, C, p, encW)
    Y = B.apnn_sumpool_fc(B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, bits, U), BS, H, Wd, C, bits,
                          B.apnn_pack(dev(Wv), p, encW), Cout, p, encW,
                          out=torch.full((BS, Cout), -7, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    sums = oracle.sumpool(Xv)
    assert np.array_equal(Y.cpu().numpy(), oracle.gemm(sums, U, 8, Wv, encW, p))
    # and it equals the two library calls it replaces
    S = B.apnn_sumpool(B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, bits, U), BS, H, Wd, C, bits, 8)
    Y2 = torch.empty((BS, Cout), dtype=torch.int32, device="cuda")
    B.apnn_layer(B.Conv(BS, 1, 1, C, Cout, 1, 1, 1, 0, p, 8, encW, U), B.apnn_pack(dev(Wv), p, encW), S, is_gemm=True, acc_out=Y2)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)


def test_sumpool_fc_refusals():
    e = torch.zeros(1 << 12, dtype=torch.int32, device="cuda")      # (refused calls launch nothing)
    for args, status in (((e, 1, 10, 10, 64, 2, e, 10, 1, P), 3),        # 300 does not fit 8 bits
                         ((e, 1, 2, 2, 48, 2, e, 10, 1, P), 1),          # channels not a multiple of 32
                         ((e, 1, 2, 2, 16384, 2, e, 10, 1, P), 2),       # too many channels
                         ((e, 1, 2, 2, 64, 2, e, 10, 2, P), 2)):         # -1/+1 with two planes
        with pytest.raises(B.ApnnError) as ei:
            B.apnn_sumpool_fc(*args, out=e)
        assert ei.value.status == status


def test_first_layer_patches_equal_convolution():
    """Input layer: 8-bit image planes x +-1 weights through the receptive-field
    packer and the matrix kernel must equal the 7x7 stride-2 convolution."""
    BS, HW, Cout = 2, 38, 64
    img = wl.image_batch(5, BS, HW)
    Wv = wl.fair_signs(6, (Cout, 3, 7, 7))
    Xp = B.apnn_pack_patches(dev(img), 7, 7, 2, 3, 8)
    Wp = B.apnn_pack_patch_weights(dev(Wv), 1, P)
    Ho = (HW + 6 - 7) // 2 + 1
    d = B.Conv(BS * Ho * Ho, 1, 1, 32 * 7, Cout, 1, 1, 1, 0, 1, 8, P, U)
    acc = torch.empty((BS * Ho * Ho, Cout), dtype=torch.int32, device="cuda")
    B.apnn_layer(d, Wp, Xp, is_gemm=True, acc_out=acc)
    torch.cuda.synchronize()
    want = oracle.conv2d(Wv, P, 1, img, U, 8, 2, 3)
    assert np.array_equal(acc.cpu().numpy().reshape(BS, Ho, Ho, Cout).transpose(0, 3, 1, 2), want)


@pytest.mark.parametrize("C,H,W,R,S,stride,pad,bits", [
    (3, 38, 38, 7, 7, 2, 3, 8),        # the input layer's geometry
    (1, 30, 41, 5, 5, 1, 2, 4),        # one channel, odd width (byte loads)
    (3, 9, 33, 3, 3, 1, 1, 2),
    (4, 19, 70, 3, 8, 3, 0, 8),        # S * C = 32 fills the word, stride 3, no padding
    (2, 21, 64, 8, 8, 2, 3, 3),        # tallest kernel
    (4, 9, 2100, 8, 8, 2, 3, 8),       # plane strings too large for LDS: general kernel
])
def test_patch_packer_geometries(C, H, W, R, S, stride, pad, bits):
    """apnn_pack_patches x apnn_pack_patch_weights through the matrix kernel equals the convolution,
    for both packer kernels and the edge geometries (overhang on every side, ragged widths)."""
    BS, Cout = 2, 40
    img = wl.uniform_codes(100 + C + W, (BS, C, H, W), bits)
    Wv = wl.fair_signs(200 + R + S, (Cout, C, R, S))
    Xp = B.apnn_pack_patches(dev(img), R, S, stride, pad, bits)
    Wp = B.apnn_pack_patch_weights(dev(Wv), 1, P)
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    d = B.Conv(BS * Ho * Wo, 1, 1, 32 * R, Cout, 1, 1, 1, 0, 1, bits, P, U)
    acc = torch.empty((BS * Ho * Wo, Cout), dtype=torch.int32, device="cuda")
    B.apnn_layer(d, Wp, Xp, is_gemm=True, acc_out=acc)
    torch.cuda.synchronize()
    want = oracle.conv2d(Wv, P, 1, img, U, bits, stride, pad)
    assert np.array_equal(acc.cpu().numpy().reshape(BS, Ho, Wo, Cout).transpose(0, 3, 1, 2), want)
    # pad words of the operand (kernel rows beyond R) are zero
    words = hp.words_u32(Xp).reshape(BS * Ho * Wo, bits, -1)
    assert (words[:, :, R:] == 0).all()


@pytest.mark.parametrize("force", ALL_FORMS)
@pytest.mark.parametrize("mode", [B.POOL_MAX2, B.POOL_SUM2])
@pytest.mark.parametrize("BS,Cin,Cout,H,Wd,R,stride,pad,with_res", [
    (2, 64, 64, 14, 14, 3, 1, 1, False),
    (1, 128, 96, 9, 11, 3, 1, 1, True),        # odd output frame: the last row and column of results are dropped
    (2, 64, 32, 12, 12, 1, 1, 0, False),       # 1 x 1
    (1, 64, 64, 56, 56, 3, 1, 1, True),        # enough rows for the 64 x 64 block tile
    (3, 32, 64, 7, 10, 3, 1, 1, True),         # one channel word: only the AND+popcount kernel has this shape
    (1, 96, 32, 13, 6, 2, 1, 1, False),        # three channel words, 2 x 2 kernel
])
def test_fused_pooling_matches_oracle(force, mode, BS, Cin, Cout, H, Wd, R, stride, pad, with_res):
    """conv -> 2 x 2 grid pooling of the int32 results -> scale/bias (+ residual) -> requantise -> repack, one kernel."""
    _force(force)
    Wv = wl.fair_signs(71 + Cin, (Cout, Cin, R, R))
    Xv = wl.uniform_codes(72 + H, (BS, Cin, H, Wd), 2)
    d = B.Conv(BS, H, Wd, Cin, Cout, R, R, stride, pad, 1, 2, P, U)
    Hp, Wp = d.Ho // 2, d.Wo // 2
    K = Cin * R * R
    div = np.sqrt(K * 3.5) * (4.0 if mode == B.POOL_SUM2 else 1.0)
    scale = (wl.normals(73, (Cout,), 1.0, 0.2) / div).astype(np.float32)
    bias = wl.normals(74, (Cout,), 1.0 if mode == B.POOL_MAX2 else 2.0, 0.3)
    res = wl.uniform_codes(75, (BS, Cout, Hp, Wp), 2) if with_res else None
    resp = B.apnn_pack_fmap(dev(res), B.LAYOUT_NCHW, 2, U) if with_res else None
    acc = torch.empty((BS, Hp, Wp, Cout), dtype=torch.int32, device="cuda")
    tf = torch.empty((BS, Hp, Wp, Cout), dtype=torch.float32, device="cuda")
    out = B.apnn_layer(d, B.apnn_pack_conv_weights(dev(Wv), 1, P), B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, 2, U),
                       q_out=2, scale=dev(scale), bias=dev(bias), residual=resp, q_res=2, res_scale=0.5,
                       acc_out=acc, float_out=tf, pool=mode)
    torch.cuda.synchronize()
    pooled = oracle.gridpool(oracle.conv2d(Wv, P, 1, Xv, U, 2, stride, pad), 2, oracle.POOL_MAX if mode == B.POOL_MAX2 else oracle.POOL_SUM)
    want_codes, want_t = oracle.epilogue(pooled, scale, bias, 2, res=res, res_scale=0.5, want_t=True)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), pooled)
    assert np.array_equal(tf.cpu().numpy().transpose(0, 3, 1, 2), want_t)
    codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), BS, Hp, Wp, Cout, 2)
    assert np.array_equal(codes, want_codes) and pad_bits == 0
    assert len(np.unique(want_codes)) == 4


def test_fused_pooling_refusals():
    e = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    f = torch.zeros(64, dtype=torch.float32, device="cuda")
    d = B.Conv(1, 8, 8, 64, 64, 3, 3, 1, 1, 1, 2, P, U)
    with pytest.raises(B.ApnnError) as ei:                      # not an apnn_pool value
        B.apnn_layer(d, e, e, q_out=2, scale=f, bias=f, pool=3)
    assert ei.value.status == 1
    with pytest.raises(B.ApnnError) as ei:                      # GEMM layers have no frame to pool
        B.apnn_layer(B.Conv(8, 1, 1, 64, 64, 1, 1, 1, 0, 1, 2, P, U), e, e, is_gemm=True, q_out=2, scale=f, bias=f, pool=1)
    assert ei.value.status == 1


@pytest.mark.parametrize("force", ["256", "128", "64", "auto"])
@pytest.mark.parametrize("q,q_out,with_res", [(2, 2, True), (4, 3, False), (1, 1, False)])
def test_fused_gemm_layer_all_matrix_tiles(force, q, q_out, with_res):
    """Fully-connected layer with the whole epilogue (scale/bias, residual, requantise, repack, int32 and fp32 side
    outputs) through every matrix-operand kernel, the large-tile one included; ragged batch."""
    B.apnn_debug_reset()
    if force != "auto":
        B.apnn_debug_force("MFMA_TILE", int(force))
    BS, K, Cout = 600, 1000, 320
    Xv = wl.uniform_codes(81 + q, (BS, K), q)
    Wv = wl.fair_signs(82, (Cout, K))
    scale = (wl.normals(83, (Cout,), 1.0, 0.2) / np.sqrt(K * ((1 << q) ** 2) / 4.0)).astype(np.float32)
    bias = wl.normals(84, (Cout,), 0.5 * (1 << q_out), 0.3)
    res = wl.uniform_codes(85, (BS, Cout), 2) if with_res else None
    d = B.Conv(BS, 1, 1, K, Cout, 1, 1, 1, 0, 1, q, P, U)
    acc = torch.empty((BS, Cout), dtype=torch.int32, device="cuda")
    tf = torch.empty((BS, Cout), dtype=torch.float32, device="cuda")
    out = B.apnn_layer(d, B.apnn_pack(dev(Wv), 1, P), B.apnn_pack(dev(Xv), q, U), is_gemm=True, q_out=q_out,
                       scale=dev(scale), bias=dev(bias),
                       residual=B.apnn_pack_fmap(dev(res.reshape(BS, Cout, 1, 1)), B.LAYOUT_NCHW, 2, U) if with_res else None,
                       q_res=2, res_scale=0.5, acc_out=acc, float_out=tf)
    torch.cuda.synchronize()
    want_acc = oracle.gemm(Xv, U, q, Wv, P, 1)
    want_codes, want_t = oracle.epilogue(want_acc, scale, bias, q_out, res=res, res_scale=0.5, want_t=True)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    assert np.array_equal(tf.cpu().numpy(), want_t)
    codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), BS, 1, 1, Cout, q_out)
    assert np.array_equal(codes.reshape(BS, Cout), want_codes) and pad_bits == 0
    assert len(np.unique(want_codes)) == (1 << q_out)


@pytest.mark.parametrize("Cin,Cout,H,with_res_a", [
    (64, 128, 28, False),      # a stage's first block: 3 x 3 stride 2 and 1 x 1 stride 2 of the same features
    (128, 256, 14, True),      # longer K for the first, short K for the second (different load depths)
    (256, 512, 7, False),      # 7 x 7 input, ragged row tiles
    (32, 64, 12, False),       # one channel word per tap: not the matrix-core kernel, launched one after the other
])
def test_layer_pair_equals_oracle(Cin, Cout, H, with_res_a):
    """apnn_layer_pair (shared launch where the dispatch allows it) against the oracle, layer by layer."""
    BS = 2
    Xv = wl.uniform_codes(70 + Cin, (BS, Cin, H, H), 2)
    Xp = B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, 2, U)
    cases = []
    for idx, (R, stride, pad) in enumerate(((3, 2, 1), (1, 2, 0))):
        Wv = wl.fair_signs(80 + idx + Cin, (Cout, Cin, R, R))
        K = Cin * R * R
        scale = (wl.normals(90 + idx, (Cout,), 1.0, 0.2) / np.sqrt(K * 3.5)).astype(np.float32)
        bias = wl.normals(95 + idx, (Cout,), 2.0, 0.3)
        d = B.Conv(BS, H, H, Cin, Cout, R, R, stride, pad, 1, 2, P, U)
        res = wl.uniform_codes(99, (BS, Cout, d.Ho, d.Wo), 2) if (with_res_a and idx == 0) else None
        out = torch.empty(B.apnn_fmap_words(BS * d.Ho * d.Wo, Cout, 2), dtype=torch.int32, device="cuda")
        acc = torch.empty((BS, d.Ho, d.Wo, Cout), dtype=torch.int32, device="cuda")
        cases.append(dict(Wv=Wv, scale=scale, bias=bias, res=res, d=d, out=out, acc=acc,
                          args=dict(d=d, W=B.apnn_pack_conv_weights(dev(Wv), 1, P), X=Xp, q_out=2, scale=dev(scale),
                                    bias=dev(bias), out=out, acc_out=acc,
                                    residual=B.apnn_pack_fmap(dev(res), B.LAYOUT_NCHW, 2, U) if res is not None else None,
                                    q_res=2, res_scale=0.5)))
    B.apnn_layer_pair(cases[0]["args"], cases[1]["args"])
    torch.cuda.synchronize()
    for c, (R, stride, pad) in zip(cases, ((3, 2, 1), (1, 2, 0))):
        d = c["d"]
        want_acc = oracle.conv2d(c["Wv"], P, 1, Xv, U, 2, stride, pad)
        want_codes, _ = oracle.epilogue(want_acc, c["scale"], c["bias"], 2, res=c["res"], res_scale=0.5)
        assert np.array_equal(c["acc"].cpu().numpy().transpose(0, 3, 1, 2), want_acc)
        codes, pad_bits = hp.unpack_fmap(hp.words_u32(c["out"]), BS, d.Ho, d.Wo, Cout, 2)
        assert np.array_equal(codes, want_codes) and pad_bits == 0


def test_layer_pair_mixed_kinds_and_validation():
    """A pair whose layers take different kernels (a large matrix layer and a small convolution) still gives both
    results; an invalid second layer fails before anything is launched."""
    Xv = wl.uniform_codes(1, (1, 64, 8, 8), 2)
    Wv = wl.fair_signs(2, (64, 64, 3, 3))
    d = B.Conv(1, 8, 8, 64, 64, 3, 3, 1, 1, 1, 2, P, U)
    acc = torch.full((1, 8, 8, 64), -5, dtype=torch.int32, device="cuda")
    conv = dict(d=d, W=B.apnn_pack_conv_weights(dev(Wv), 1, P), X=B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, 2, U), acc_out=acc)
    A = wl.uniform_codes(3, (300, 256), 2)
    Wm = wl.fair_signs(4, (200, 256))
    dm = B.Conv(300, 1, 1, 256, 200, 1, 1, 1, 0, 1, 2, P, U)
    accm = torch.empty((300, 200), dtype=torch.int32, device="cuda")
    Lm = B.LayerDesc(dm.c(), 1, 0, None, None, None, 0, 0.0, accm.data_ptr(), None, 0)
    Lc = B.LayerDesc(d.c(), 0, 0, None, None, None, 0, 0.0, acc.data_ptr(), None, 0)
    Wmp, Amp = B.apnn_pack(dev(Wm), 1, P), B.apnn_pack(dev(A), 2, U)
    import ctypes as C
    st = torch.cuda.current_stream().cuda_stream
    rc = B.lib().apnn_layer_pair(C.byref(Lm), Wmp.data_ptr(), Amp.data_ptr(), None,
                                 C.byref(Lc), conv["W"].data_ptr(), conv["X"].data_ptr(), None, st)
    torch.cuda.synchronize()
    assert rc == 0
    assert np.array_equal(accm.cpu().numpy(), oracle.gemm(Wm, P, 1, A, U, 2).T)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), oracle.conv2d(Wv, P, 1, Xv, U, 2, 1, 1))
    # second description invalid (Cin not a multiple of 32): nothing runs, the first output stays as it was
    acc.fill_(-5)
    bad = B.Conv(1, 8, 8, 48, 64, 3, 3, 1, 1, 1, 2, P, U)
    Lb = B.LayerDesc(bad.c(), 0, 0, None, None, None, 0, 0.0, acc.data_ptr(), None, 0)
    rc = B.lib().apnn_layer_pair(C.byref(Lc), conv["W"].data_ptr(), conv["X"].data_ptr(), None,
                                 C.byref(Lb), conv["W"].data_ptr(), conv["X"].data_ptr(), None, st)
    torch.cuda.synchronize()
    assert rc == 1 and (acc.cpu().numpy() == -5).all()
