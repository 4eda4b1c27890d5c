"""Seeded random sweep of apnn_layer over shapes, encodings, bit widths, outputs, residuals, pooling and kernel
choices, against the oracle: meant to reach the corners the hand-picked cases miss (ragged tiles on every side,
block tiles that reach beyond M or N, one-plane outputs, eight-plane outputs, residuals of any width)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2106_12169_amd import binding as B
from paper_2106_12169_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu
U, P = B.ENC_UNSIGNED, B.ENC_PM1
FORCES = ("auto", "auto", "auto", "64", "32split1", "32split4", "32chunked", "pop4", "pop2", "128", "32split1wide2")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _force(force):
    B.apnn_debug_reset()
    if force.startswith("pop"):
        B.apnn_debug_force("MFMA", 0)
        B.apnn_debug_force("TILE", int(force[3:]))
    elif force == "32chunked":
        B.apnn_debug_force("MFMA_TILE", 32)
        B.apnn_debug_force("MFMA_SMALL", 0)
    elif force.startswith("32split"):
        B.apnn_debug_force("MFMA_TILE", 32)
        B.apnn_debug_force("MFMA_NSPLIT", int(force[7]))
        if "wide" in force:
            B.apnn_debug_force("MFMA_FN", int(force[-1]))
    elif force != "auto":
        B.apnn_debug_force("MFMA_TILE", int(force))


def _draw(rng):
    c = dict()
    c["force"] = FORCES[rng.integers(len(FORCES))]
    c["BS"] = int(rng.integers(1, 4))
    c["Cin"] = int(rng.choice([32, 64, 64, 96, 128, 192]))
    c["Cout"] = int(rng.choice([32, 64, 96, 128, 160]))
    c["R"] = int(rng.choice([1, 3, 3, 5]))
    c["S"] = c["R"] if rng.integers(3) else int(rng.choice([1, 2, 3]))
    c["stride"] = int(rng.choice([1, 1, 2, 3]))
    c["pad"] = int(rng.integers(0, max(c["R"], c["S"]) // 2 + 2))
    c["H"] = int(rng.integers(max(1, c["R"] - 2 * c["pad"]), 19))
    c["W"] = int(rng.integers(max(1, c["S"] - 2 * c["pad"]), 23))
    kind = rng.integers(4)
    c["encW"], c["p"] = (P, 1) if kind < 2 else (U, int(rng.integers(1, 4)))
    c["encX"], c["q"] = (P, 1) if rng.integers(6) == 0 else (U, int(rng.integers(1, 5)))
    c["q_out"] = int(rng.choice([0, 1, 2, 2, 2, 3, 4, 8]))
    c["q_res"] = int(rng.integers(1, 9)) if (c["q_out"] and rng.integers(2)) else 0
    c["pool"] = int(rng.choice([0, 0, 0, 1, 2]))
    return c


@pytest.mark.parametrize("seed", range(int(os.environ.get("APNN_RANDOM_SEEDS", "60"))))   # more seeds for a longer hunt
def test_random_layer(seed):
    rng = np.random.default_rng(7000 + seed)
    c = _draw(rng)
    _force(c["force"])
    BS, Cin, Cout, H, W, R, S = c["BS"], c["Cin"], c["Cout"], c["H"], c["W"], c["R"], c["S"]
    stride, pad, p, q, encW, encX = c["stride"], c["pad"], c["p"], c["q"], c["encW"], c["encX"]
    Wv = wl.operand(seed, Cout, Cin * R * S, p, encW).reshape(Cout, Cin, R, S)
    Xv = wl.operand(seed + 1, BS * Cin, H * W, q, encX).reshape(BS, Cin, H, W)
    d = B.Conv(BS, H, W, Cin, Cout, R, S, stride, pad, p, q, encW, encX)
    Ho, Wo = d.Ho, d.Wo
    pool = c["pool"] if (Ho >= 2 and Wo >= 2) else 0
    Hq, Wq = (Ho // 2, Wo // 2) if pool else (Ho, Wo)
    q_out, q_res = c["q_out"], c["q_res"]
    K = Cin * R * S
    amp = ((1 << p) - 1 if encW == U else 1) * ((1 << q) - 1 if encX == U else 1) * (4 if pool == 2 else 1)
    scale = (wl.normals(seed + 2, (Cout,), 1.0, 0.3) * (1 << max(q_out, 1)) / (np.sqrt(K) * amp + 1)).astype(np.float32)
    bias = wl.normals(seed + 3, (Cout,), 0.4 * (1 << max(q_out, 1)), 0.5)
    res = wl.uniform_codes(seed + 4, (BS, Cout, Hq, Wq), q_res) if q_res else None
    acc = torch.full((BS, Hq, Wq, Cout), -7, dtype=torch.int32, device="cuda")
    tf = torch.full((BS, Hq, Wq, Cout), -7.0, dtype=torch.float32, device="cuda")
    kw = dict(acc_out=acc, pool=pool)
    if q_out:
        kw.update(q_out=q_out, scale=dev(scale), bias=dev(bias), float_out=tf)
        if q_res:
            kw.update(residual=B.apnn_pack_fmap(dev(res), B.LAYOUT_NCHW, q_res, U), q_res=q_res, res_scale=0.37)
    # nothing here is refused: every form of the product computes -1/+1 features and fused pooling
    out = B.apnn_layer(d, B.apnn_pack_conv_weights(dev(Wv), p, encW), B.apnn_pack_fmap(dev(Xv), B.LAYOUT_NCHW, q, encX), **kw)
    torch.cuda.synchronize()
    want_acc = oracle.conv2d(Wv, encW, p, Xv, encX, q, stride, pad)
    if pool:
        want_acc = oracle.gridpool(want_acc, 2, oracle.POOL_MAX if pool == B.POOL_MAX2 else oracle.POOL_SUM)
    assert np.array_equal(acc.cpu().numpy().transpose(0, 3, 1, 2), want_acc), c
    if q_out:
        want_codes, want_t = oracle.epilogue(want_acc, scale, bias, q_out, res=res, res_scale=0.37, want_t=True)
        assert np.array_equal(tf.cpu().numpy().transpose(0, 3, 1, 2), want_t), c
        codes, pad_bits = hp.unpack_fmap(hp.words_u32(out), BS, Hq, Wq, Cout, q_out)
        assert np.array_equal(codes, want_codes) and pad_bits == 0, c


def test_sweep_reaches_every_form():
    """The draws cover pooled layers and -1/+1 features on the AND+popcount kernel as well as on the matrix core."""
    seen = set()
    for seed in range(60):
        c = _draw(np.random.default_rng(7000 + seed))
        seen.add((c["force"].startswith("pop"), bool(c["pool"]), c["encX"] == P))
    assert {(True, True, False), (True, False, True), (False, True, False), (False, False, True)} <= seen, seen
