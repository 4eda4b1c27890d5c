"""GPU parity of the input layer (8-bit image, few channels, 8-bit integer matrix
instruction) against the oracle's convolution and epilogue, through the C-ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2106_12169_amd import binding as B
from paper_2106_12169_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu
U, P = B.ENC_UNSIGNED, B.ENC_PM1


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _weights(seed, shape, p, enc):
    return wl.fair_signs(seed, shape) if enc == P else wl.uniform_codes(seed, shape, p)


@pytest.mark.parametrize("C,H,W,R,S,stride,pad,bits,Cout,p,enc", [
    (3, 38, 38, 7, 7, 2, 3, 8, 64, 1, P),      # the network's input layer geometry
    (1, 30, 41, 5, 5, 1, 2, 4, 40, 1, P),      # one channel, odd width, ragged channel tile
    (3, 9, 33, 3, 3, 1, 1, 2, 32, 1, P),
    (4, 19, 70, 3, 8, 3, 0, 8, 128, 3, U),     # S = 8 fills a K segment; unsigned weights; four channel tiles
    (2, 21, 64, 8, 8, 2, 3, 8, 96, 7, U),      # widest weights, three channel tiles
    (4, 20, 24, 8, 5, 1, 2, 8, 64, 1, P),      # K of 8 steps: more than one batch of loads
    (3, 12, 8, 3, 3, 1, 4, 8, 64, 1, P),       # narrowest frame; windows entirely left and right of it
    (3, 10, 300, 2, 7, 5, 1, 8, 33, 1, P),     # stride 5, one channel beyond a tile
    (3, 67, 67, 11, 11, 4, 2, 8, 64, 1, P),    # 11 x 11 stride 4 (the first layer of an AlexNet-shaped network): two segments per kernel row
    (2, 23, 40, 3, 9, 1, 4, 8, 32, 2, U),      # S = 9: one byte in the second segment
    (1, 17, 16, 2, 16, 2, 7, 6, 96, 1, P),     # S = 16 = the frame width: windows mostly outside
])
def test_input_layer_accumulators(C, H, W, R, S, stride, pad, bits, Cout, p, enc):
    BS = 2
    img = wl.uniform_codes(300 + C + W, (BS, C, H, W), bits)
    Wv = _weights(400 + R + S, (Cout, C, R, S), p, enc)
    Wp = B.apnn_pack_input_weights(dev(Wv), p, enc)
    d = B.Conv(BS, H, W, C, Cout, R, S, stride, pad, p, bits, enc, U)
    acc = torch.full((BS, d.Ho, d.Wo, Cout), -7, dtype=torch.int32, device="cuda")
    B.apnn_input_layer(d, Wp, dev(img), acc_out=acc)
    torch.cuda.synchronize()
    want = oracle.conv2d(Wv, enc, p, img, U, bits, stride, pad)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), want)


@pytest.mark.parametrize("bits", [1, 3, 5, 7])
def test_input_layer_ignores_image_bits_above_q(bits):
    """conv.q is the number of significant image bits: bytes with higher bits set give the product of the low
    `bits` bits, as the plane packers do (they ignore higher bits as well)."""
    BS, C, H, W, Cout = 2, 3, 20, 37, 64
    raw = wl.uniform_codes(310 + bits, (BS, C, H, W), 8)
    assert (raw >> bits).max() > 0
    low = (raw & ((1 << bits) - 1)).astype(np.uint8)
    Wv = wl.fair_signs(410 + bits, (Cout, C, 5, 5))
    d = B.Conv(BS, H, W, C, Cout, 5, 5, 2, 2, 1, bits, P, U)
    acc = torch.empty((BS, d.Ho, d.Wo, Cout), dtype=torch.int32, device="cuda")
    B.apnn_input_layer(d, B.apnn_pack_input_weights(dev(Wv), 1, P), dev(raw), acc_out=acc)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), oracle.conv2d(Wv, P, 1, low, U, bits, 2, 2))


@pytest.mark.parametrize("q_out,with_res", [(2, False), (2, True), (1, False), (8, False)])
def test_input_layer_fused_epilogue(q_out, with_res):
    BS, HW, Cout = 2, 38, 64
    img = wl.image_batch(5, BS, HW)
    Wv = wl.fair_signs(6, (Cout, 3, 7, 7))
    d = B.Conv(BS, HW, HW, 3, Cout, 7, 7, 2, 3, 1, 8, P, U)
    scale = (wl.normals(7, (Cout,), 1.0, 0.2) / 800.0).astype(np.float32)
    bias = wl.normals(8, (Cout,), 0.5 * (1 << q_out), 0.3)
    res = wl.uniform_codes(9, (BS, Cout, d.Ho, d.Wo), 2) if with_res else None
    resp = B.apnn_pack_fmap(dev(res), B.LAYOUT_NCHW, 2, U) if with_res else None
    acc = torch.empty((BS, d.Ho, d.Wo, Cout), dtype=torch.int32, device="cuda")
    tf = torch.empty((BS, d.Ho, d.Wo, Cout), dtype=torch.float32, device="cuda")
    out = B.apnn_input_layer(d, B.apnn_pack_input_weights(dev(Wv), 1, P), dev(img), q_out=q_out, scale=dev(scale),
                             bias=dev(bias), residual=resp, q_res=2, res_scale=0.5, acc_out=acc, float_out=tf)
    torch.cuda.synchronize()
    want_acc = oracle.conv2d(Wv, P, 1, img, U, 8, 2, 3)
    want_codes, want_t = oracle.epilogue(want_acc, scale, bias, q_out, res=res, res_scale=0.5, want_t=True)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), want_acc)
    got_t = tf.cpu().numpy().transpose(0, 3, 1, 2)
    assert np.allclose(got_t, want_t, rtol=1e-5, atol=0) and np.array_equal(got_t, want_t)
    codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), BS, d.Ho, d.Wo, Cout, q_out)
    assert np.array_equal(codes, want_codes) and pad_bits == 0
    if q_out <= 2:
        assert len(np.unique(want_codes)) == (1 << q_out)


def test_input_layer_equals_patch_path_at_full_size():
    """224 x 224 batch 8 (the launch the network bench times): the packed codes equal those of the
    receptive-field packer + matrix kernel path, which the oracle covers at this size in the network test;
    sampled accumulators are compared with the oracle directly."""
    layers = wl.resnet18_layers()
    L = layers[0]
    wv, sc, bi = wl.network_params(layers)[L.name]
    img = wl.image_batch(2004, 8, 224)
    d = B.Conv(8, L.H, L.W, L.Cin, L.Cout, L.R, L.S, L.stride, L.pad, L.p, L.q, P, U)
    acc = torch.empty((8, d.Ho, d.Wo, L.Cout), dtype=torch.int32, device="cuda")
    out = B.apnn_input_layer(d, B.apnn_pack_input_weights(dev(wv), L.p, P), dev(img), q_out=L.q_out, scale=dev(sc),
                             bias=dev(bi), acc_out=acc)
    torch.cuda.synchronize()
    got = acc.cpu().numpy()
    rng = np.random.default_rng(11)
    x = img.astype(np.int64)
    w = wv.astype(np.int64)
    for _ in range(400):
        n, ho, wo, co = rng.integers(8), rng.integers(d.Ho), rng.integers(d.Wo), rng.integers(L.Cout)
        if _ < 8:                                           # the corners of the first and last image
            n, ho, wo = (0, 7)[_ & 1], (0, d.Ho - 1)[(_ >> 1) & 1], (0, d.Wo - 1)[(_ >> 2) & 1]
        s = 0
        for r in range(L.R):
            for t in range(L.S):
                h, ww = ho * L.stride + r - L.pad, wo * L.stride + t - L.pad
                if 0 <= h < L.H and 0 <= ww < L.W:
                    s += int((w[co, :, r, t] * x[n, :, h, ww]).sum())
        assert got[n, ho, wo, co] == s, (n, ho, wo, co)
    want_codes, _ = oracle.epilogue(got.transpose(0, 3, 1, 2), sc, bi, L.q_out)
    codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), 8, d.Ho, d.Wo, L.Cout, L.q_out)
    assert np.array_equal(codes, want_codes) and pad_bits == 0


def test_input_layer_refusals():
    img = dev(wl.uniform_codes(1, (1, 3, 16, 16), 8))
    acc = torch.empty((1, 16, 16, 64), dtype=torch.int32, device="cuda")

    def status(fn):
        with pytest.raises(B.ApnnError) as e:
            fn()
        return e.value.status

    w17 = dev(wl.fair_signs(2, (64, 3, 3, 17)))
    assert status(lambda: B.apnn_pack_input_weights(w17, 1, P)) == 2                # S > 16
    w8 = dev(wl.uniform_codes(3, (64, 3, 3, 3), 8))
    assert status(lambda: B.apnn_pack_input_weights(w8, 8, U)) == 2                 # 8-bit weights
    Wp = B.apnn_pack_input_weights(dev(wl.fair_signs(4, (64, 3, 3, 3))), 1, P)
    assert status(lambda: B.apnn_input_layer(B.Conv(1, 16, 16, 3, 192, 3, 3, 1, 1, 1, 8, P, U), Wp, img, acc_out=acc)) == 2
    assert status(lambda: B.apnn_input_layer(B.Conv(1, 16, 7, 3, 64, 3, 3, 1, 1, 1, 8, P, U), Wp, img, acc_out=acc)) == 2
    assert status(lambda: B.apnn_input_layer(B.Conv(1, 16, 16, 3, 64, 3, 3, 1, 1, 1, 8, P, P), Wp, img, acc_out=acc)) in (1, 2)
    assert status(lambda: B.apnn_input_layer(B.Conv(1, 16, 16, 3, 64, 3, 3, 1, 1, 1, 8, P, U), Wp, img)) == 1   # no output
    # 7-bit weights with a K beyond the exact range
    assert status(lambda: B.apnn_input_layer(B.Conv(1, 16, 16, 16, 64, 8, 8, 1, 1, 7, 8, U, U), Wp, img, acc_out=acc)) == 2


@pytest.mark.parametrize("seed", range(int(__import__("os").environ.get("APNN_RANDOM_SEEDS", "40"))))
def test_random_input_layer(seed):
    """Seeded random geometries: the unaligned 8-byte segments, their clamped start and the shifted-in zeros on
    both sides of the frame, ragged channel tiles and row tiles, every plane count."""
    rng = np.random.default_rng(5000 + seed)
    C, R, S = int(rng.integers(1, 5)), int(rng.integers(1, 9)), int(rng.integers(1, 9))
    stride, pad = int(rng.integers(1, 5)), int(rng.integers(0, 5))
    H = int(rng.integers(max(1, R - 2 * pad), 30))
    W = int(rng.integers(max(8, S - 2 * pad), 60))
    bits = int(rng.integers(1, 9))
    Cout = int(rng.choice([32, 40, 64, 96, 128, 7]))
    enc, p = (P, 1) if rng.integers(2) else (U, int(rng.integers(1, 8)))
    q_out = int(rng.choice([0, 1, 2, 3, 8])) if Cout % 32 == 0 else 0
    BS = int(rng.integers(1, 4))
    img = wl.uniform_codes(seed, (BS, C, H, W), bits)
    Wv = _weights(seed + 1, (Cout, C, R, S), p, enc)
    d = B.Conv(BS, H, W, C, Cout, R, S, stride, pad, p, bits, enc, U)
    acc = torch.full((BS, d.Ho, d.Wo, Cout), -7, dtype=torch.int32, device="cuda")
    K = C * R * S
    wmax = 1 if enc == P else (1 << p) - 1
    scale = (wl.normals(seed + 2, (Cout,), 1.0, 0.3) * (1 << max(q_out, 1)) / (np.sqrt(K) * wmax * ((1 << bits) - 1) + 1)).astype(np.float32)
    bias = wl.normals(seed + 3, (Cout,), 0.4 * (1 << max(q_out, 1)), 0.5)
    kw = dict(acc_out=acc)
    if q_out:
        kw.update(q_out=q_out, scale=dev(scale), bias=dev(bias))
    out = B.apnn_input_layer(d, B.apnn_pack_input_weights(dev(Wv), p, enc), dev(img), **kw)
    torch.cuda.synchronize()
    want = oracle.conv2d(Wv, enc, p, img, U, bits, stride, pad)
    case = (C, H, W, R, S, stride, pad, bits, Cout, p, enc, q_out)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), want), case
    if q_out:
        want_codes, _ = oracle.epilogue(want, scale, bias, q_out)
        codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), BS, d.Ho, d.Wo, Cout, q_out)
        assert np.array_equal(codes, want_codes) and pad_bits == 0, case
