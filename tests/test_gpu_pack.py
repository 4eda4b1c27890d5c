"""GPU parity of the bit-plane packers: bit-exact against the source codes
(decoded from the packed words with numpy) and zero pad bits."""
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


@pytest.mark.parametrize("rows,K,bits,enc", [
    (128, 128, 1, P), (128, 128, 2, U), (37, 203, 3, U), (5, 31, 8, U), (300, 1000, 5, U),
    (64, 4096, 2, U), (1, 1, 1, U), (33, 96, 1, P), (7, 48, 4, U),
])
def test_pack_matrix(rows, K, bits, enc):
    src = wl.operand(100 + rows + K, rows, K, bits, enc)
    words = hp.words_u32(B.apnn_pack(dev(src), bits, enc))
    codes, pad = hp.unpack_matrix(words, rows, K, bits)
    want = hp.pm1_to_bits(src) if enc == P else src
    assert np.array_equal(codes, want)
    assert pad == 0 and words.size == B.apnn_packed_words(rows, K, bits)


def test_pack_ignores_bits_above_the_declared_width():
    src = wl.uniform_codes(5, (9, 70), 8)
    codes, _ = hp.unpack_matrix(hp.words_u32(B.apnn_pack(dev(src), 3, U)), 9, 70, 3)
    assert np.array_equal(codes, src & 7)


@pytest.mark.parametrize("layout", [B.LAYOUT_NHWC, B.LAYOUT_NCHW])
@pytest.mark.parametrize("N,C,H,W,bits", [(2, 64, 5, 7, 2), (1, 128, 9, 9, 2), (3, 32, 4, 4, 3), (1, 96, 6, 5, 1),
                                          (2, 64, 8, 8, 8), (1, 96, 6, 6, 2), (2, 40, 4, 6, 3), (3, 160, 28, 28, 2)])
def test_pack_fmap(layout, N, C, H, W, bits):
    nchw = wl.uniform_codes(7, (N, C, H, W), bits)
    src = nchw if layout == B.LAYOUT_NCHW else nchw.transpose(0, 2, 3, 1)
    words = hp.words_u32(B.apnn_pack_fmap(dev(src), layout, bits, U))
    codes, pad = hp.unpack_fmap(words, N, H, W, C, bits)
    assert np.array_equal(codes, nchw) and pad == 0


@pytest.mark.parametrize("layout", [B.LAYOUT_NHWC, B.LAYOUT_NCHW])
@pytest.mark.parametrize("N,C,H,W", [(2, 64, 4, 6), (1, 96, 5, 5), (2, 40, 8, 2)])
def test_pack_fmap_pm1(layout, N, C, H, W):
    nchw = wl.fair_signs(8, (N, C, H, W))
    src = nchw if layout == B.LAYOUT_NCHW else nchw.transpose(0, 2, 3, 1)
    words = hp.words_u32(B.apnn_pack_fmap(dev(src), layout, 1, P))
    codes, pad = hp.unpack_fmap(words, N, H, W, C, 1)
    assert np.array_equal(codes, hp.pm1_to_bits(nchw)) and pad == 0


def test_pack_conv_weights_layout():
    Cout, Cin, R, S = 5, 64, 3, 3
    w = wl.fair_signs(3, (Cout, Cin, R, S))
    words = hp.words_u32(B.apnn_pack_conv_weights(dev(w), 1, P))
    Cw = Cin // 32
    # [Cout][bits][R][S][Cw]: row (co, r, s) holds the channels of that tap
    codes, pad = hp.unpack_planes(words, Cout * R * S, Cin, 1, Cw)
    assert np.array_equal(codes.reshape(Cout, R, S, Cin), hp.pm1_to_bits(w).transpose(0, 2, 3, 1)) and pad == 0
    w2 = wl.uniform_codes(4, (Cout, Cin, R, S), 3)
    words = hp.words_u32(B.apnn_pack_conv_weights(dev(w2), 3, U)).reshape(Cout, 3, R * S, Cw)
    for t in range(3):
        plane, _ = hp.unpack_planes(words[:, t].reshape(-1), Cout * R * S, Cin, 1, Cw)
        assert np.array_equal(plane.reshape(Cout, R, S, Cin), ((w2 >> t) & 1).transpose(0, 2, 3, 1))


@pytest.mark.parametrize("rows,K", [(19, 333), (5, 256), (3, 1), (7, 31), (2, 1000), (64, 4096)])
@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_quantize_matches_oracle(bits, rows, K):
    x = wl.normals(9, (rows, K), 2.0, 3.0)
    special = [np.nan, np.inf, -np.inf, 0.0, -0.0, 1e30][:K]
    x[0, :len(special)] = special
    zero, step = -0.75, 0.37
    words = hp.words_u32(B.apnn_quantize(dev(x), zero, step, bits))
    codes, pad = hp.unpack_matrix(words, rows, K, bits)
    assert np.array_equal(codes, oracle.quantize(x, zero, step, bits)) and pad == 0
