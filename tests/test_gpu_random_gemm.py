"""Seeded random sweep of apnn_gemm over ragged shapes, bit widths, encodings and kernel choices, against the
oracle (bit-exact)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2106_12169_amd import binding as B
from paper_2106_12169_amd import workloads as wl

pytestmark = pytest.mark.gpu
U, P = B.ENC_UNSIGNED, B.ENC_PM1
FORCES = ("auto", "auto", "256", "256", "128", "128", "64", "32split1", "32split4", "32chunked", "pop8", "pop4", "pop2")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("seed", range(int(os.environ.get("APNN_RANDOM_SEEDS", "50"))))   # more seeds for a longer hunt
def test_random_gemm(seed):
    rng = np.random.default_rng(9000 + seed)
    force = FORCES[rng.integers(len(FORCES))]
    B.apnn_debug_reset()
    if force.startswith("pop"):
        B.apnn_debug_force("MFMA", 0)
        B.apnn_debug_force("TILE", int(force[3:]))
    elif force == "32chunked":
        B.apnn_debug_force("MFMA_TILE", 32)
        B.apnn_debug_force("MFMA_SMALL", 0)
    elif force.startswith("32split"):
        B.apnn_debug_force("MFMA_TILE", 32)
        B.apnn_debug_force("MFMA_NSPLIT", int(force[-1]))
    elif force != "auto":
        B.apnn_debug_force("MFMA_TILE", int(force))
    M, N = int(rng.integers(1, 420)), int(rng.integers(1, 420))
    K = int(rng.choice([rng.integers(1, 70), rng.integers(70, 700), rng.integers(700, 2100)]))
    encW, p = (P, 1) if rng.integers(2) else (U, int(rng.integers(1, 9)))
    encX, q = (P, 1) if rng.integers(4) == 0 else (U, int(rng.integers(1, 9)))
    i8 = int(rng.integers(4))                       # 2, 3: the 8-bit integer matrix forms (outputs / K shared out among the waves)
    if i8 >= 2 and not force.startswith("pop"):
        B.apnn_debug_force("INT8", i8)
    Wv, Xv = wl.operand(seed, M, K, p, encW), wl.operand(seed + 1, N, K, q, encX)
    Y = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    B.apnn_gemm(B.apnn_pack(dev(Wv), p, encW), B.apnn_pack(dev(Xv), q, encX), M, N, K, p, q, encW, encX, out=Y)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), oracle.gemm(Wv, encW, p, Xv, encX, q)), (force, i8, M, N, K, p, q, encW, encX)
