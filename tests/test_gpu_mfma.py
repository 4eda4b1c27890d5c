"""GPU parity of the FP4 matrix-core GEMM path against the integer oracle,
bit-exact, at sizes that span several K chunks, ragged tails in M, N and K, every
digit-kind pair and multi-digit (more than two bits) operands."""
import numpy as np
import pytest
import torch

import oracle
from paper_2106_12169_amd import binding as B
from paper_2106_12169_amd import workloads as wl

pytestmark = pytest.mark.gpu
U, P = wl.ENC_UNSIGNED, wl.ENC_PM1


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.fixture(autouse=True, params=["32", "32split1", "32split4", "32chunked", "64", "128", "256"])
def mfma_tile(request):
    B.apnn_debug_force("MFMA", -1)
    B.apnn_debug_force("MFMA_SMALL", -1)
    B.apnn_debug_force("MFMA_TILE", int(request.param[:2] if request.param.startswith("32") else request.param))
    B.apnn_debug_force("MFMA_NSPLIT", -1)
    if request.param == "32chunked":
        B.apnn_debug_force("MFMA_SMALL", 0)
    if request.param.startswith("32split"):
        B.apnn_debug_force("MFMA_NSPLIT", int(request.param[-1]))


def gpu_gemm(W, encW, p, X, encX, q):
    M, K = W.shape
    N = X.shape[0]
    Y = B.apnn_gemm(B.apnn_pack(dev(W), p, encW), B.apnn_pack(dev(X), q, encX), M, N, K, p, q, encW, encX)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


KINDS = [(U, 1), (U, 2), (P, 1)]


@pytest.mark.parametrize("encW,p", KINDS)
@pytest.mark.parametrize("encX,q", KINDS)
@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (300, 520, 1000), (70, 33, 257), (513, 257, 4096 + 32)])
def test_mfma_gemm_matches_oracle(encW, p, encX, q, M, N, K):
    W = wl.operand(7 * M + K + p, M, K, p, encW)
    X = wl.operand(9 * N + K + q, N, K, q, encX)
    assert np.array_equal(gpu_gemm(W, encW, p, X, encX, q), oracle.gemm(W, encW, p, X, encX, q))


@pytest.mark.parametrize("p,q,K", [(3, 5, 1000), (2, 8, 777), (8, 8, 250), (5, 1, 4096), (4, 4, 2048), (7, 3, 300)])
def test_mfma_multi_digit_operands(p, q, K):
    M, N = 150, 290
    W = wl.uniform_codes(3 * p + K, (M, K), p)
    X = wl.uniform_codes(5 * q + K, (N, K), q)
    assert np.array_equal(gpu_gemm(W, U, p, X, U, q), oracle.gemm(W, U, p, X, U, q))
    if q == 1:
        Xs = wl.fair_signs(77, (N, K))
        assert np.array_equal(gpu_gemm(W, U, p, Xs, P, 1), oracle.gemm(W, U, p, Xs, P, 1))


def test_mfma_extremes():
    K = 3000
    W = np.full((260, K), 3, np.uint8)
    assert (gpu_gemm(W, U, 2, W, U, 2) == 9 * K).all()
    ones = np.ones((260, K), np.int8)
    assert (gpu_gemm(ones, P, 1, -ones, P, 1) == -K).all()
    assert (gpu_gemm(-ones, P, 1, W, U, 2) == -3 * K).all()
    W8 = np.full((70, 255), 255, np.uint8)                 # largest 8-bit accumulators that stay exact
    assert (gpu_gemm(W8, U, 8, W8, U, 8) == 255 * 255 * 255).all()


def test_mfma_falls_back_when_fp32_would_not_be_exact():
    """K * 3 * 3 >= 2^24: the dispatcher must take the integer kernel; the result stays exact."""
    K = 1 << 21
    W = np.full((4, K), 3, np.uint8)
    assert (gpu_gemm(W, U, 2, W, U, 2) == 9 * K).all()
