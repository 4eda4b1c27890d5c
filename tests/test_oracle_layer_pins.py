"""Pins for the oracle's convolution, quantiser, fused epilogue and pooling."""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import network as onet
from paper_2106_12169_amd import workloads as wl

U, P = wl.ENC_UNSIGNED, wl.ENC_PM1


@pytest.mark.parametrize("Cin,Cout,H,Wd,R,stride,pad,encW,p,q", [
    (5, 4, 9, 7, 3, 1, 1, P, 1, 2),
    (3, 6, 12, 12, 7, 2, 3, P, 1, 8),      # first-layer shape family
    (8, 5, 8, 8, 1, 2, 0, P, 1, 2),        # 1x1 stride-2 shortcut
    (4, 3, 10, 6, 3, 2, 1, U, 2, 3),
    (2, 2, 5, 5, 5, 1, 2, U, 3, 1),
])
def test_conv_vs_float64_library(Cin, Cout, H, Wd, R, stride, pad, encW, p, q):
    BS = 2
    W = wl.operand(21, Cout, Cin * R * R, p, encW).reshape(Cout, Cin, R, R)
    X = wl.uniform_codes(22, (BS, Cin, H, Wd), q)
    Y = oracle.conv2d(W, encW, p, X, U, q, stride, pad)
    ref = F.conv2d(torch.from_numpy(X.astype(np.float64)), torch.from_numpy(W.astype(np.float64)),
                   stride=stride, padding=pad)
    assert Y.shape == tuple(ref.shape)
    assert np.array_equal(Y, ref.numpy().astype(np.int64))


def test_conv_pm1_features_zero_padding():
    """+-1 features: taps outside the frame must add 0, not -1 (Sec. 4.2 (b))."""
    W = wl.fair_signs(1, (3, 4, 3, 3))
    X = wl.fair_signs(2, (1, 4, 5, 5))
    Y = oracle.conv2d(W, P, 1, X, P, 1, 1, 1)
    ref = F.conv2d(torch.from_numpy(X.astype(np.float64)), torch.from_numpy(W.astype(np.float64)), padding=1)
    assert np.array_equal(Y, ref.numpy().astype(np.int64))


def test_conv_1x1_is_gemm():
    BS, Cin, Cout, H = 2, 19, 6, 4
    W = wl.fair_signs(3, (Cout, Cin, 1, 1))
    X = wl.uniform_codes(4, (BS, Cin, H, H), 2)
    Y = oracle.conv2d(W, P, 1, X, U, 2, 1, 0)
    rows = X.transpose(0, 2, 3, 1).reshape(-1, Cin)                      # pixel-major rows
    G = oracle.gemm(W.reshape(Cout, Cin), P, 1, rows, U, 2)              # Cout x pixels
    assert np.array_equal(Y, G.reshape(Cout, BS, H, H).transpose(1, 0, 2, 3))


def test_conv_all_ones_counts_in_frame_taps():
    C, H = 6, 5
    W = np.ones((1, C, 3, 3), np.uint8)
    X = np.ones((1, C, H, H), np.uint8)
    Y = oracle.conv2d(W, U, 1, X, U, 1, 1, 1)[0, 0]
    assert Y[2, 2] == 9 * C and Y[0, 2] == 6 * C and Y[2, 0] == 6 * C and Y[0, 0] == 4 * C and Y[4, 4] == 4 * C


def test_conv_equals_im2col_gemm():
    BS, Cin, Cout, H, R, stride, pad = 2, 3, 4, 7, 3, 2, 1
    W = wl.fair_signs(5, (Cout, Cin, R, R))
    X = wl.uniform_codes(6, (BS, Cin, H, H), 2)
    Y = oracle.conv2d(W, P, 1, X, U, 2, stride, pad)
    Xp = np.pad(X, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    Ho = (H + 2 * pad - R) // stride + 1
    cols = np.empty((BS, Ho, Ho, Cin, R, R), np.uint8)
    for ho in range(Ho):
        for wo in range(Ho):
            cols[:, ho, wo] = Xp[:, :, ho * stride:ho * stride + R, wo * stride:wo * stride + R]
    G = oracle.gemm(W.reshape(Cout, -1), P, 1, cols.reshape(BS * Ho * Ho, -1), U, 2)
    assert np.array_equal(Y, G.reshape(Cout, BS, Ho, Ho).transpose(1, 0, 2, 3))


def test_conv_one_hot_weight_shifts_image():
    """A single tap at (r, s) of channel c copies the shifted image: checks the tap/offset signs."""
    H = 6
    X = wl.uniform_codes(8, (1, 2, H, H), 3)
    for (r, s) in [(0, 0), (0, 2), (2, 1), (1, 1)]:
        W = np.zeros((1, 2, 3, 3), np.uint8)
        W[0, 1, r, s] = 1
        Y = oracle.conv2d(W, U, 1, X, U, 3, 1, 1)[0, 0]
        Xp = np.pad(X[0, 1].astype(np.int32), 1)
        assert np.array_equal(Y, Xp[r:r + H, s:s + H])


# ---- quantiser ----------------------------------------------------------------

def test_quantize_closed_forms():
    z, s = np.float32(0.5), np.float32(0.25)
    k = np.arange(-3, 20)
    x = (z + k * s).astype(np.float32)                                  # exactly representable
    assert oracle.quantize(x, z, s, 3).tolist() == np.clip(k, 0, 7).tolist()
    x2 = np.nextafter(x, np.float32(-np.inf))                           # just below each step
    assert oracle.quantize(x2, z, s, 3).tolist() == np.clip(k - 1, 0, 7).tolist()
    assert oracle.quantize(np.array([np.nan, -np.inf, np.inf], np.float32), 0.0, 1.0, 2).tolist() == [0, 0, 3]
    with pytest.raises(oracle.OracleError):
        oracle.quantize(x, 0.0, 0.0, 2)


def test_quantize_matches_exact_rational_floor_away_from_steps():
    x = wl.normals(5, (4000,), 1.0, 3.0)
    z, s, bits = np.float32(-0.3), np.float32(0.7), 4
    got = oracle.quantize(x, z, s, bits)
    for xi, g in zip(x[:500], got[:500]):
        v = (Fraction(float(xi)) - Fraction(float(z))) / Fraction(float(s))
        if abs(v - round(v)) < Fraction(1, 10000):
            continue
        assert g == min(max(v.numerator // v.denominator, 0), 15)


# ---- fused epilogue -----------------------------------------------------------

def _is_correctly_rounded(exact: Fraction, r: np.float32) -> bool:
    lo, hi = np.nextafter(r, np.float32(-np.inf)), np.nextafter(r, np.float32(np.inf))
    d = abs(exact - Fraction(float(r)))
    return d <= abs(exact - Fraction(float(lo))) and d <= abs(exact - Fraction(float(hi)))


def test_epilogue_single_fma_is_correctly_rounded():
    C, HW = 8, 50
    Y = (wl.raw_u64(7, 0, C * HW) % np.uint64(60001)).astype(np.int64) - 30000
    Y = Y.astype(np.int32).reshape(1, C, HW)
    scale, bias = wl.normals(8, (C,), 0, 0.01), wl.normals(9, (C,), 1.5, 0.1)
    codes, t = oracle.epilogue(Y, scale, bias, 2, want_t=True)
    for c in range(C):
        for i in range(HW):
            exact = Fraction(float(scale[c])) * int(Y[0, c, i]) + Fraction(float(bias[c]))
            assert _is_correctly_rounded(exact, t[0, c, i])
            f = np.floor(t[0, c, i])
            assert codes[0, c, i] == min(max(f, 0), 3)


def test_epilogue_boundaries_and_residual():
    # scale 0.5, bias 0: Y = 2k lands exactly on integer k; Y = 2k-1 on k - 0.5 -> floor k-1
    Y = np.arange(-4, 12, dtype=np.int32).reshape(1, 1, -1)
    codes, t = oracle.epilogue(Y, [0.5], [0.0], 2, want_t=True)
    assert t.ravel().tolist() == (np.arange(-4, 12) * 0.5).tolist()
    assert codes.ravel().tolist() == [0, 0, 0, 0, 0, 0, 1, 1, 2, 2, 3, 3, 3, 3, 3, 3]
    # -0.0 and tiny negatives clamp to 0 (ReLU)
    codes, _ = oracle.epilogue(np.array([[[0, -1]]], np.int32), [1e-30], [-0.0], 2)
    assert codes.ravel().tolist() == [0, 0]
    # residual: t = res_scale * res + (a*Y + b)
    Y = np.array([[[2, 2, 2, 2]]], np.int32)
    res = np.array([[[0, 1, 2, 3]]], np.uint8)
    codes, t = oracle.epilogue(Y, [0.25], [0.25], 3, res=res, res_scale=0.5, want_t=True)
    assert t.ravel().tolist() == [0.75, 1.25, 1.75, 2.25]
    assert codes.ravel().tolist() == [0, 1, 1, 2]
    # per-channel parameters are indexed by the channel axis (axis 1), not by pixel
    Y = np.ones((2, 3, 4), np.int32)
    codes, _ = oracle.epilogue(Y, [1.0, 2.0, 3.0], [0.0, 0.0, 0.0], 2)
    assert (codes[:, 0] == 1).all() and (codes[:, 1] == 2).all() and (codes[:, 2] == 3).all()


def test_folded_bn_equals_fused_formula_of_sec_5_2():
    """floor(max(BN(x) - z, 0) / s) evaluated in double == folded single-fma epilogue,
    for inputs whose quotient is not within 1e-3 of an integer."""
    C, n = 6, 400
    g = 1.0 + 0.3 * wl.normals(1, (C,)).astype(np.float64)
    b = wl.normals(2, (C,)).astype(np.float64)
    mu = 10 * wl.normals(3, (C,)).astype(np.float64)
    var = np.abs(50 + 20 * wl.normals(4, (C,)).astype(np.float64)) + 1.0
    eps, z, s, q = 1e-5, 0.25, 0.4, 3
    scale, bias = oracle.fold_bn(g, b, mu, var, eps, z, s)
    Y = ((wl.raw_u64(5, 0, C * n) % np.uint64(201)).astype(np.int64) - 100).astype(np.int32).reshape(1, C, n)
    codes, _ = oracle.epilogue(Y, scale, bias, q)
    x = Y[0].astype(np.float64)
    bn = (x - mu[:, None]) / np.sqrt(var[:, None] + eps) * g[:, None] + b[:, None]
    v = np.maximum(bn - z, 0.0) / s
    safe = (np.abs(v - np.round(v)) > 1e-3) | (bn - z < -1e-3)     # clamped negatives are safely 0
    want = np.clip(np.floor(v), 0, (1 << q) - 1)
    assert safe.mean() > 0.9 and len(np.unique(want[safe])) == 8
    assert np.array_equal(codes[0][safe], want[safe].astype(np.uint8))


# ---- pooling ---------------------------------------------------------------

def test_maxpool_vs_library_and_sumpool():
    X = wl.uniform_codes(3, (2, 3, 9, 11), 2)
    got = oracle.maxpool(X, 3, 2, 1)
    ref = F.max_pool2d(torch.from_numpy(X.astype(np.float32)), 3, 2, 1).numpy()
    assert np.array_equal(got, ref.astype(np.uint8))
    got = oracle.maxpool(X, 2, 2, 0)
    ref = F.max_pool2d(torch.from_numpy(X.astype(np.float32)), 2, 2, 0).numpy()
    assert np.array_equal(got, ref.astype(np.uint8))
    S = oracle.sumpool(X[:, :, :7, :7])
    assert np.array_equal(S, X[:, :, :7, :7].astype(np.int64).sum((2, 3)))
    with pytest.raises(oracle.OracleError):
        oracle.sumpool(np.full((1, 1, 10, 10), 3, np.uint8))            # 300 does not fit 8 bits


# ---- chained network: self-consistency of the wiring ---------------------------

def test_small_residual_network_runs_and_uses_all_levels():
    layers = wl.resnet18_layers(image_hw=32, num_classes=10, widths=(32, 32, 64, 64))
    params = wl.network_params(layers)
    img = wl.image_batch(77, 2, 32)
    out = onet.run(layers, params, img)
    assert out["fc"].shape == (2, 10) and out["fc"].dtype == np.int32
    for L in layers:
        if L.kind == "conv":
            hist = np.bincount(out[L.name].ravel(), minlength=4) / out[L.name].size
            assert hist.min() > (0.002 if L.name == 'conv1' else 0.05), (L.name, hist)
    # the shortcut enters the epilogue: dropping it must change the block output
    L = next(l for l in layers if l.name == "s1b1_conv2")
    w, sc, bi = params[L.name]
    acc = oracle.conv2d(w, P, 1, out[L.src], U, 2, 1, 1)
    with_res, _ = oracle.epilogue(acc, sc, bi, 2, res=out[L.res], res_scale=L.res_scale)
    without, _ = oracle.epilogue(acc, sc, bi, 2)
    assert np.array_equal(with_res, out[L.name]) and not np.array_equal(without, out[L.name])


def test_gridpool_vs_library_and_by_hand():
    """Grid pooling of int32 results: hand example, library max / average pooling, dropped ragged edges."""
    Y = np.array([[[[1, -5, 7, 2, 9],
                    [3, 4, -8, 0, 9],
                    [-1, -2, 6, 6, 9],
                    [-3, -4, 5, 7, 9],
                    [100, 100, 100, 100, 100]]]], np.int32)             # 5 x 5: last row and column are dropped
    assert oracle.gridpool(Y, 2, oracle.POOL_MAX).tolist() == [[[[4, 7], [-1, 7]]]]
    assert oracle.gridpool(Y, 2, oracle.POOL_SUM).tolist() == [[[[3, 1], [-10, 24]]]]
    rng = np.random.default_rng(5)
    Z = rng.integers(-3000, 3000, (2, 3, 12, 10)).astype(np.int32)
    zt = torch.from_numpy(Z.astype(np.float64))
    for k in (2, 3):
        want_max = torch.nn.functional.max_pool2d(zt, k, k).numpy()
        want_sum = torch.nn.functional.avg_pool2d(zt, k, k).numpy() * (k * k)
        assert np.array_equal(oracle.gridpool(Z, k, oracle.POOL_MAX), want_max.astype(np.int32))
        assert np.array_equal(oracle.gridpool(Z, k, oracle.POOL_SUM), np.rint(want_sum).astype(np.int32))
    assert np.array_equal(oracle.gridpool(Z, 1, oracle.POOL_MAX), Z) and np.array_equal(oracle.gridpool(Z, 1, oracle.POOL_SUM), Z)
    with pytest.raises(oracle.OracleError):                               # sums must fit int32
        oracle.gridpool(np.full((1, 1, 2, 2), 2**30, np.int32), 2, oracle.POOL_SUM)
