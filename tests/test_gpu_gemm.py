"""GPU parity of apnn_gemm against the integer oracle: bit-exact int32."""
import os

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


def gpu_gemm(W, encW, p, X, encX, q):
    M, K = W.shape
    N = X.shape[0]
    Wp, Xp = B.apnn_pack(dev(W), p, encW), B.apnn_pack(dev(X), q, encX)
    Y = B.apnn_gemm(Wp, Xp, M, N, K, p, q, encW, encX)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


@pytest.fixture(params=["auto", "pop8", "pop4", "pop2", "mfma32", "mfma32split1", "mfma32split4", "mfma32chunked", "mfma64", "mfma128", "mfma256"])
def tile(request):
    """Kernel path under test: the library's own choice, the AND+popcount kernel with
    each register tile, or the FP4 matrix-core kernel with each block tile."""
    B.apnn_debug_reset()
    kind = request.param
    if kind.startswith("pop"):
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


CASES = [
    # encW, p, encX, q, M, N, K
    (P, 1, U, 2, 128, 128, 128),          # benchmark configuration 0
    (U, 1, U, 1, 130, 70, 200),
    (P, 1, U, 2, 257, 131, 1000),         # several tiles, ragged M/N/K tails
    (U, 2, U, 2, 96, 160, 513),
    (U, 1, U, 4, 64, 64, 2048),
    (U, 3, U, 5, 50, 90, 777),
    (U, 2, U, 8, 33, 47, 300),
    (U, 8, U, 8, 20, 20, 4000),
    (P, 1, P, 1, 140, 150, 999),          # Case II (XOR), K not a multiple of 32
    (U, 4, P, 1, 75, 129, 640),           # mirrored Case III
    (P, 1, U, 8, 129, 65, 96),
    (U, 1, U, 1, 1, 1, 1),
    (P, 1, U, 2, 3, 1000, 64),            # FC-like thin shapes
]


@pytest.mark.parametrize("encW,p,encX,q,M,N,K", CASES)
def test_gemm_matches_oracle(tile, encW, p, encX, q, M, N, K):
    W = wl.operand(11 * M + K, M, K, p, encW)
    X = wl.operand(13 * N + K, N, K, q, encX)
    got = gpu_gemm(W, encW, p, X, encX, q)
    assert np.array_equal(got, oracle.gemm(W, encW, p, X, encX, q))


def test_gemm_extremes_and_empty():
    K = 700
    W = np.full((40, K), 255, np.uint8)
    assert (gpu_gemm(W, U, 8, W, U, 8) == K * 255 * 255).all()        # largest accumulators
    Z = np.zeros((40, K), np.uint8)
    assert (gpu_gemm(W, U, 8, Z, U, 8) == 0).all()
    ones = np.ones((40, K), np.int8)
    assert (gpu_gemm(ones, P, 1, -ones, P, 1) == -K).all()
    # K = 0 writes zeros; M = 0 / N = 0 write nothing
    Y = torch.full((4, 5), 7, dtype=torch.int32, device="cuda")
    e = torch.empty(1, dtype=torch.int32, device="cuda")
    B.apnn_gemm(e, e, 4, 5, 0, 1, 2, P, U, out=Y)
    assert (Y.cpu().numpy() == 0).all()
    Y.fill_(7)
    B.apnn_gemm(e, e, 0, 5, 64, 1, 2, P, U, out=Y)
    assert (Y.cpu().numpy() == 7).all()


def test_gemm_is_deterministic():
    wk = wl.gemm_w1a2(512, 0)
    a = gpu_gemm(wk.weights(), P, 1, wk.activations(), U, 2)
    b = gpu_gemm(wk.weights(), P, 1, wk.activations(), U, 2)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("w,a", wl.SWEEP_BITS)
def test_sweep_reduced_size(w, a):
    wk = wl.sweep_workload(w, a, 384)
    W, X = wk.weights(), wk.activations()
    assert np.array_equal(gpu_gemm(W, U, w, X, U, a), oracle.gemm(W, U, w, X, U, a))


def test_config1_full_size_every_element():
    """4096^3 in the launch configuration the benchmark times: every one of the 4096 x 4096 outputs against the
    oracle, plus size-independent properties."""
    wk = wl.CONFIG1
    W, X = wk.weights(), wk.activations()
    Y = gpu_gemm(W, wk.encW, wk.p, X, wk.encX, wk.q)
    assert np.array_equal(Y, oracle.gemm(W, wk.encW, wk.p, X, wk.encX, wk.q))
    # parity of every entry: sum of K odd/even terms -> Y = rowsum(X) (mod 2)
    assert np.array_equal(Y & 1, np.broadcast_to(X.astype(np.int64).sum(1) & 1, Y.shape))
    # column sums: sum_m Y[m][n] = sum_k (sum_m W[m][k]) X[n][k]
    colw = W.astype(np.int64).sum(0)
    assert np.array_equal(Y.astype(np.int64).sum(0), X.astype(np.int64) @ colw)


def test_config1_full_size_popcount_kernel_every_element():
    """The same product on the plane-pair AND + popcount kernel (the literal emulation of Sec. 3), every element."""
    B.apnn_debug_force("MFMA", 0)
    wk = wl.CONFIG1
    W, X = wk.weights(), wk.activations()
    Y = gpu_gemm(W, wk.encW, wk.p, X, wk.encX, wk.q)
    assert np.array_equal(Y, oracle.gemm(W, wk.encW, wk.p, X, wk.encX, wk.q))


@pytest.mark.parametrize("w,a", wl.SWEEP_BITS)
def test_config2_full_size_every_element(w, a):
    wk = wl.sweep_workload(w, a)
    W, X = wk.weights(), wk.activations()
    Y = gpu_gemm(W, U, w, X, U, a)
    assert np.array_equal(Y, oracle.gemm(W, U, w, X, U, a))


@pytest.mark.parametrize("w,a", wl.PAPER_FC_BITS)
@pytest.mark.parametrize("dim", wl.PAPER_FC_DIMS)
def test_paper_fc_shapes(w, a, dim):
    """Fully-connected shapes of the paper's APMM evaluation (batch 64, K = N = dim), default dispatch."""
    wk = wl.paper_fc_workload(w, a, dim)
    W, X = wk.weights(), wk.activations()
    assert np.array_equal(gpu_gemm(W, U, w, X, U, a), oracle.gemm(W, U, w, X, U, a))


@pytest.mark.parametrize("encW,p,encX,q,K", [
    (U, 3, U, 5, 4096),            # 2 x 3 base-4 digit passes, weights of Eq. 1 carried by the instruction's block scales
    (P, 1, P, 1, 4096 + 40),       # Case II on the large-tile kernel, K pad correction
    (U, 2, P, 1, 2000),            # mirrored Case III, ragged K
])
def test_large_tile_kernel_full_width_sampled(encW, p, encX, q, K):
    """M = N = 4096 (256 tiles of 256 x 256, the launch shape of the headline benchmark) for other digit kinds:
    sampled rows against the oracle plus the column-sum identity over every output."""
    M = N = 4096
    W = wl.operand(900 + p + K, M, K, p, encW)
    X = wl.operand(901 + q + K, N, K, q, encX)
    Y = gpu_gemm(W, encW, p, X, encX, q)
    rows = np.unique(np.concatenate([[0, 255, 256, 4095], (wl.raw_u64(7, 0, 12) % np.uint64(M)).astype(int)]))
    assert np.array_equal(Y[rows], oracle.gemm(W[rows], encW, p, X, encX, q))
    colw = W.astype(np.int64).sum(0)
    assert np.array_equal(Y.astype(np.int64).sum(0), X.astype(np.int64) @ colw)


@pytest.mark.parametrize("force,M,N,K", [
    ("128", 256, 512, 96),         # 2 x 4 tiles: one tile per region
    ("128", 250, 1000, 333),       # the same grid doubled in N, ragged on every side
    ("128", 1024, 1536, 160),      # 8 x 12 tiles: regions of 4 x 3
    ("256", 1024, 2048, 64),       # 4 x 8 tiles of 256
    ("256", 512, 1000, 200),       # 2 x 4, ragged N
])
def test_large_tile_kernel_region_order(force, M, N, K):
    """Tile grids that divide into 2 x 4 regions are walked region by region (one per XCD): every tile must still be
    computed exactly once, whatever the grid."""
    B.apnn_debug_reset()
    B.apnn_debug_force("MFMA_TILE", int(force))
    W = wl.operand(700 + M, M, K, 1, P)
    X = wl.operand(701 + N, N, K, 2, U)
    Y = gpu_gemm(W, P, 1, X, U, 2)
    assert np.array_equal(Y, oracle.gemm(W, P, 1, X, U, 2))


@pytest.mark.parametrize("force,M,N,K", [
    ("128", 257, 131, 1000),       # one row into the third row of tiles
    ("256", 257, 131, 1000),
    ("128", 2000, 2048, 96),       # a shape the library's own choice sends to this kernel: 80 rows short of a tile
    ("256", 4000, 4096, 64),
    ("auto", 2000, 2048, 96),
    ("64", 257, 131, 1000),
    ("32", 257, 131, 1000),
    ("pop4", 257, 131, 1000),
])
def test_ragged_m_writes_nothing_beyond_the_output(force, M, N, K):
    """The rows of the last tile that lie beyond M must not be stored anywhere: the output is the first M rows of a
    larger buffer whose remaining rows hold a sentinel."""
    if force.startswith("pop"):
        B.apnn_debug_force("MFMA", 0)
        B.apnn_debug_force("TILE", int(force[3:]))
    elif force != "auto":
        B.apnn_debug_force("MFMA_TILE", int(force))
    W = wl.operand(800 + M, M, K, 1, P)
    X = wl.operand(801 + N, N, K, 2, U)
    guard = 300
    buf = torch.full((M + guard, N), -123456789, dtype=torch.int32, device="cuda")
    B.apnn_gemm(B.apnn_pack(dev(W), 1, P), B.apnn_pack(dev(X), 2, U), M, N, K, 1, 2, P, U, out=buf[:M])
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    assert (got[M:] == -123456789).all()
    assert np.array_equal(got[:M], oracle.gemm(W, P, 1, X, U, 2))
