"""Pins for the integer oracle (GEMM side): printed examples, closed forms,
invariants, a float64 library cross-check and the bit-plane identity."""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2106_12169_amd import workloads as wl

U, P = wl.ENC_UNSIGNED, wl.ENC_PM1


def _parse_rows(txt, dtype):
    return np.array([[int(v) for v in row.split()] for row in txt.split(";")], dtype=dtype)


def _golden_cases(path):
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, ew, p, ex, q, w, x, y = [f.strip() for f in line.split("|")]
        encW, encX = (P if ew == "P" else U), (P if ex == "P" else U)
        yield (name, encW, int(p), encX, int(q),
               _parse_rows(w, np.int8 if encW == P else np.uint8),
               _parse_rows(x, np.int8 if encX == P else np.uint8),
               _parse_rows(y, np.int32))


def test_printed_examples(golden_dir):
    cases = list(_golden_cases(os.path.join(golden_dir, "apbit_examples.txt")))
    assert len(cases) >= 8
    for name, encW, p, encX, q, W, X, Y in cases:
        assert np.array_equal(oracle.gemm(W, encW, p, X, encX, q), Y), name
        assert np.array_equal(oracle.apbit_gemm(W, encW, p, X, encX, q), Y), name


def test_decode():
    assert oracle.decode(np.array([1, -1, 1], np.int8), 1, P).tolist() == [1, -1, 1]
    assert oracle.decode(np.array([0, 5, 7], np.uint8), 3, U).tolist() == [0, 5, 7]
    assert oracle.decode(np.array([255], np.uint8), 8, U).tolist() == [255]
    with pytest.raises(oracle.OracleError):
        oracle.decode(np.array([0], np.int8), 1, P)          # 0 is not a +-1 value
    with pytest.raises(oracle.OracleError):
        oracle.decode(np.array([4], np.uint8), 2, U)         # does not fit 2 bits
    with pytest.raises(oracle.OracleError):
        oracle.decode(np.array([1], np.int8), 2, P)          # +-1 is defined for 1 bit only


@pytest.mark.parametrize("p,q", [(1, 1), (1, 2), (2, 1), (2, 2)])
def test_brute_force_tiny(p, q):
    """Every operand pair for K <= 3, M = N = 1, against integer arithmetic on tuples."""
    for K in (1, 2, 3):
        for w in itertools.product(range(1 << p), repeat=K):
            for x in itertools.product(range(1 << q), repeat=K):
                want = sum(a * b for a, b in zip(w, x))
                got = oracle.gemm(np.array([w], np.uint8), U, p, np.array([x], np.uint8), U, q)
                assert got[0, 0] == want


def test_brute_force_signs():
    for K in (1, 2, 3, 4):
        for w in itertools.product((-1, 1), repeat=K):
            for x in itertools.product(range(4), repeat=K):
                want = sum(a * b for a, b in zip(w, x))
                W, X = np.array([w], np.int8), np.array([x], np.uint8)
                assert oracle.gemm(W, P, 1, X, U, 2)[0, 0] == want
                assert oracle.gemm(X, U, 2, W, P, 1)[0, 0] == want
            for x in itertools.product((-1, 1), repeat=K):
                want = sum(a * b for a, b in zip(w, x))
                assert oracle.gemm(np.array([w], np.int8), P, 1, np.array([x], np.int8), P, 1)[0, 0] == want


@pytest.mark.parametrize("p,q,K", [(1, 2, 37), (3, 5, 100), (8, 8, 33), (2, 8, 64)])
def test_closed_forms(p, q, K):
    M, N = 5, 7
    X = wl.uniform_codes(11, (N, K), q)
    Wmax = np.full((M, K), (1 << p) - 1, np.uint8)
    Xmax = np.full((N, K), (1 << q) - 1, np.uint8)
    assert (oracle.gemm(Wmax, U, p, Xmax, U, q) == K * ((1 << p) - 1) * ((1 << q) - 1)).all()
    rowsum = X.astype(np.int64).sum(1)
    ones = np.ones((M, K), np.int8)
    assert np.array_equal(oracle.gemm(ones, P, 1, X, U, q), np.tile(rowsum, (M, 1)))
    assert np.array_equal(oracle.gemm(-ones, P, 1, X, U, q), -np.tile(rowsum, (M, 1)))
    assert (oracle.gemm(Wmax, U, p, np.zeros((N, K), np.uint8), U, q) == 0).all()
    onehot = np.zeros((K, K), np.uint8)
    onehot[np.arange(K), np.arange(K)] = 1
    assert np.array_equal(oracle.gemm(onehot, U, 1, X, U, q), X.T.astype(np.int32))   # picks column k


def test_orientation_is_not_symmetric():
    """Y is M x N with W supplying rows: a transposed operand or output must fail."""
    W = wl.uniform_codes(1, (3, 9), 2)
    X = wl.uniform_codes(2, (4, 9), 3)
    Y = oracle.gemm(W, U, 2, X, U, 3)
    assert Y.shape == (3, 4)
    assert np.array_equal(Y, oracle.gemm(X, U, 3, W, U, 2).T)
    assert Y[1, 2] == int(W[1].astype(int) @ X[2].astype(int))


@pytest.mark.parametrize("encW,p,encX,q", [(U, 1, U, 1), (P, 1, U, 2), (U, 2, U, 2), (U, 1, U, 4),
                                            (U, 3, U, 5), (U, 2, U, 8), (P, 1, P, 1), (U, 8, P, 1),
                                            (P, 1, U, 8), (U, 7, U, 6)])
def test_float64_library_crosscheck_and_identity(encW, p, encX, q):
    M, N, K = 13, 17, 203                       # K spans several words and a ragged tail
    W = wl.operand(5, M, K, p, encW)
    X = wl.operand(6, N, K, q, encX)
    Y = oracle.gemm(W, encW, p, X, encX, q)
    Wd = torch.from_numpy(W.astype(np.float64))
    Xd = torch.from_numpy(X.astype(np.float64))
    assert np.array_equal(Y, (Wd @ Xd.T).numpy().astype(np.int64))
    # "Y = WX mathematically": the bit-plane emulation must agree with the plain product
    assert np.array_equal(Y, oracle.apbit_gemm(W, encW, p, X, encX, q))


def test_plane_linearity_and_k_permutation():
    M, N, K, q = 6, 5, 77, 4
    W = wl.fair_signs(3, (M, K))
    X = wl.uniform_codes(4, (N, K), q)
    Y = oracle.gemm(W, P, 1, X, U, q)
    lo = oracle.gemm(W, P, 1, X & 1, U, 1)
    hi = oracle.gemm(W, P, 1, X >> 1, U, q - 1)
    assert np.array_equal(Y, lo + 2 * hi)
    perm = np.argsort(wl.raw_u64(9, 0, K))
    assert np.array_equal(Y, oracle.gemm(W[:, perm], P, 1, X[:, perm], U, q))


def test_overflow_is_reported():
    K = 40000
    W = np.full((1, K), 255, np.uint8)
    with pytest.raises(oracle.OracleError) as e:
        oracle.gemm(W, U, 8, W, U, 8)          # 40000 * 255^2 > 2^31
    assert e.value.code == 3


def test_rows_variant_matches():
    W = wl.fair_signs(1, (9, 50))
    X = wl.uniform_codes(2, (4, 50), 2)
    full = oracle.gemm(W, P, 1, X, U, 2)
    assert np.array_equal(oracle.gemm_rows(W, P, 1, X, U, 2, 3, 7), full[3:7])


def test_config1_statistics_on_a_row_sample():
    """+-1 fair weights x uniform 2-bit activations (mean 1.5, variance 1.25): over n,
    row m of Y has mean 1.5 * sum_k w[m][k] and variance 1.25 K."""
    wk = wl.CONFIG1
    W, X = wk.weights()[:64], wk.activations()
    Y = oracle.gemm(W, wk.encW, wk.p, X, wk.encX, wk.q).astype(np.float64)
    sigma = np.sqrt(1.25 * wk.K)
    want_mean = 1.5 * W.astype(np.float64).sum(1)
    assert np.abs(Y.mean(1) - want_mean).max() < 6 * sigma / np.sqrt(wk.N)
    assert abs((Y - Y.mean(1, keepdims=True)).std() / sigma - 1.0) < 0.01
