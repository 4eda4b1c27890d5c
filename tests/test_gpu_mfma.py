"""GPU parity of the FP4 matrix-core GEMM path (operands of at most two bits)
against the integer oracle, bit-exact, at sizes that span several K chunks,
ragged tails in M, N and K, and every operand-kind pair."""
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


@pytest.fixture(autouse=True)
def force_mfma(monkeypatch):
    monkeypatch.setenv("APNN_MFMA", "2")


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


def test_mfma_extremes():
    K = 3000
    W = np.full((260, K), 3, np.uint8)
    assert (gpu_gemm(W, U, 2, W, U, 2) == 9 * K).all()
    ones = np.ones((260, K), np.int8)
    assert (gpu_gemm(ones, P, 1, -ones, P, 1) == -K).all()
    assert (gpu_gemm(-ones, P, 1, W, U, 2) == -3 * K).all()


def test_mfma_falls_back_when_fp32_would_not_be_exact(monkeypatch):
    """K * 3 * 3 >= 2^24: the dispatcher must take the integer kernel; the result stays exact."""
    K = 1 << 21
    W = np.full((4, K), 3, np.uint8)
    assert (gpu_gemm(W, U, 2, W, U, 2) == 9 * K).all()
