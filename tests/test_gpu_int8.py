"""GPU parity of the single-pass 8-bit integer matrix form of the product (operands of more than two bits,
Sec. 6.1.1) against the integer oracle, bit-exact: every (p, q) up to 8 bits, the -1/+1 encodings, ragged tails in
M, N and K, the largest accumulators, the fused epilogue, and the cases only this form computes on the matrix unit
(K beyond the exact range of the FP4 form)."""
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


# INT8 override: 2 = the kernel that shares the outputs out among the waves of a block, 3 = the one that shares K out
# (where it has an instance: at most 10 planes in all, not both operands above four), 1 = the library's choice of them
FORMS = [2, 3]


def gpu_gemm(W, encW, p, X, encX, q, force=1):
    M, K = W.shape
    N = X.shape[0]
    if force:
        B.apnn_debug_force("INT8", force)
    Y = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    B.apnn_gemm(B.apnn_pack(dev(W), p, encW), B.apnn_pack(dev(X), q, encX), M, N, K, p, q, encW, encX, out=Y)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("p", range(1, 9))
@pytest.mark.parametrize("q", range(1, 9))
def test_every_bit_width_pair(p, q, form):
    M, N, K = 150, 290, 777                               # two row tiles, three column tiles, K not a multiple of 128
    W = wl.uniform_codes(3 * p + K, (M, K), p)
    X = wl.uniform_codes(5 * q + K, (N, K), q)
    assert np.array_equal(gpu_gemm(W, U, p, X, U, q, form), oracle.gemm(W, U, p, X, U, q))


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("q", range(1, 9))
@pytest.mark.parametrize("K", [64, 1000])
def test_pm1_against_every_width_both_ways(q, K, form):
    """Case III and its mirror on this form: twice the sum of the 0/1 plane less the other operand's row sums."""
    M, N = 130, 129
    S = wl.fair_signs(40 + q, (M, K))
    X = wl.uniform_codes(50 + q, (N, K), q)
    assert np.array_equal(gpu_gemm(S, P, 1, X, U, q, form), oracle.gemm(S, P, 1, X, U, q))
    assert np.array_equal(gpu_gemm(X, U, q, S, P, 1, form), oracle.gemm(X, U, q, S, P, 1))
    if q == 1:
        T = wl.fair_signs(60, (N, K))
        assert np.array_equal(gpu_gemm(S, P, 1, T, P, 1, form), oracle.gemm(S, P, 1, T, P, 1))     # Case II as well


@pytest.mark.parametrize("M,N,K,p,q", [
    (20, 20, 4000, 8, 8),          # beyond the exact range of the FP4 form: 4000 * 255 * 255 >= 2^24
    (257, 131, 33, 8, 8),          # one chunk, mostly padding
    (384, 512, 2048, 3, 5),        # whole tiles (regions of tiles per XCD), the sweep's bit widths
    (512, 1024, 1024, 2, 8),
    (1, 1, 1, 8, 8),
    (300, 1, 129, 5, 7),
    (256, 384, 4096 + 100, 8, 2),  # long K: many groups per wave, ragged last group
    (130, 140, 128 * 5, 4, 4),     # an odd number of chunks
])
@pytest.mark.parametrize("form", [1] + FORMS)
def test_shapes(M, N, K, p, q, form):
    W = wl.uniform_codes(71 + M + p, (M, K), p)
    X = wl.uniform_codes(72 + N + q, (N, K), q)
    assert np.array_equal(gpu_gemm(W, U, p, X, U, q, form), oracle.gemm(W, U, p, X, U, q))


@pytest.mark.parametrize("form", FORMS)
def test_extremes(form):
    K = 3000
    W = np.full((140, K), 255, np.uint8)
    assert (gpu_gemm(W, U, 8, W, U, 8, form) == K * 255 * 255).all()          # largest accumulators
    Z = np.zeros((140, K), np.uint8)
    assert (gpu_gemm(W, U, 8, Z, U, 8, form) == 0).all() and (gpu_gemm(Z, U, 8, W, U, 8, form) == 0).all()
    H = np.full((140, K), 128, np.uint8)                                  # the byte -128 + 128: both offsets at once
    assert (gpu_gemm(H, U, 8, H, U, 8, form) == K * 128 * 128).all()
    ones = np.ones((140, K), np.int8)
    assert (gpu_gemm(-ones, P, 1, W, U, 8, form) == -255 * K).all()
    K2 = 33024                                                            # the longest K the int32 result allows at 8 x 8 bits
    W2 = np.full((3, K2), 255, np.uint8)
    assert (gpu_gemm(W2, U, 8, W2, U, 8, form) == K2 * 255 * 255).all()


def test_taken_when_the_fp4_form_would_not_be_exact():
    """Library's own choice: K * 3 * 3 >= 2^24, and a small 8 x 8-bit product with K = 4000."""
    K = 1 << 21
    W = np.full((4, K), 3, np.uint8)
    assert (gpu_gemm(W, U, 2, W, U, 2, force=False) == 9 * K).all()
    W8 = wl.uniform_codes(5, (20, 4000), 8)
    assert np.array_equal(gpu_gemm(W8, U, 8, W8, U, 8, force=False), oracle.gemm(W8, U, 8, W8, U, 8))


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("M,N", [(257, 131), (2000, 256)])
def test_ragged_m_writes_nothing_beyond_the_output(M, N, form):
    K = 500
    W = wl.uniform_codes(91, (M, K), 3)
    X = wl.uniform_codes(92, (N, K), 5)
    B.apnn_debug_force("INT8", form)
    buf = torch.full((M + 200, N), -123456789, dtype=torch.int32, device="cuda")
    B.apnn_gemm(B.apnn_pack(dev(W), 3, U), B.apnn_pack(dev(X), 5, U), M, N, K, 3, 5, U, U, out=buf[:M])
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    assert (got[M:] == -123456789).all() and np.array_equal(got[:M], oracle.gemm(W, U, 3, X, U, 5))


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("q,q_out,with_res,encW,p", [(5, 2, True, P, 1), (8, 3, False, U, 3), (4, 8, False, U, 4)])
def test_fused_layer(q, q_out, with_res, encW, p, form):
    """Fully connected layer with the whole epilogue (scale/bias, residual, requantise, repack, int32 and fp32 side
    outputs) on this form; ragged batch."""
    B.apnn_debug_force("INT8", form)
    BS, K, Cout = 600, 1000, 320
    Xv = wl.uniform_codes(81 + q, (BS, K), q)
    Wv = wl.operand(82, Cout, K, p, encW)
    wmax = 1 if encW == P else (1 << p) - 1
    scale = (wl.normals(83, (Cout,), 1.0, 0.2) / (wmax * np.sqrt(K * ((1 << q) ** 2) / 4.0))).astype(np.float32)
    bias = (wl.normals(84, (Cout,), 0.5 * (1 << q_out), 0.3)
            - (0 if encW == P else scale * K * wmax / 2 * ((1 << q) - 1) / 2)).astype(np.float32)
    res = wl.uniform_codes(85, (BS, Cout), 2) if with_res else None
    d = B.Conv(BS, 1, 1, K, Cout, 1, 1, 1, 0, p, q, encW, U)
    acc = torch.empty((BS, Cout), dtype=torch.int32, device="cuda")
    tf = torch.empty((BS, Cout), dtype=torch.float32, device="cuda")
    out = B.apnn_layer(d, B.apnn_pack(dev(Wv), p, encW), B.apnn_pack(dev(Xv), q, U), is_gemm=True, q_out=q_out,
                       scale=dev(scale), bias=dev(bias),
                       residual=B.apnn_pack_fmap(dev(res.reshape(BS, Cout, 1, 1)), B.LAYOUT_NCHW, 2, U) if with_res else None,
                       q_res=2, res_scale=0.5, acc_out=acc, float_out=tf)
    torch.cuda.synchronize()
    want_acc = oracle.gemm(Xv, U, q, Wv, encW, p)
    want_codes, want_t = oracle.epilogue(want_acc, scale, bias, q_out, res=res, res_scale=0.5, want_t=True)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    got_t = tf.cpu().numpy()
    assert np.allclose(got_t, want_t, rtol=1e-5, atol=0) and np.array_equal(got_t, want_t)
    codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), BS, 1, 1, Cout, q_out)
    assert np.array_equal(codes.reshape(BS, Cout), want_codes) and pad_bits == 0
    assert len(np.unique(want_codes)) >= min(1 << q_out, 4)
