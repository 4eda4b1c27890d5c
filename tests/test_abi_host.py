"""Host-side checks that need no GPU: the library loads, exports every symbol
the header declares, computes sizes, validates arguments before touching the
device, and folds batch-norm parameters like the oracle does."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2106_12169_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a 16-byte aligned non-null "device pointer" that must never be dereferenced


def _declared(*headers):
    out = set()
    for h in headers:
        text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", h)).read(), flags=re.S)
        out |= set(re.findall(r"\b(apnn_[a-z0-9_]+)\s*\(", text))
    return out


def test_library_exports_every_declared_symbol():
    from paper_2106_12169_amd import bench_probes as BP
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["apnn.h", "apnn_bench.h", "apnn_debug.h"]
    declared = _declared("apnn.h", "apnn_debug.h")
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    L = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    probes = _declared("apnn_bench.h")
    assert probes == set(BP.EXPORTS)
    LB = C.CDLL(BP.LIB_PATH)
    for name in probes:
        assert hasattr(LB, name) and not hasattr(L, name), name


def test_workspace_is_never_needed_and_overrides_are_host_only():
    assert B.apnn_workspace_bytes(B.Conv(8, 28, 28, 128, 128, 3, 3, 1, 1), q_out=2) == 0
    assert B.lib().apnn_workspace_bytes(None) == 0
    B.apnn_debug_force("MFMA", 0)
    B.apnn_debug_force("MFMA", -1)
    with pytest.raises(B.ApnnError) as ei:
        B.apnn_debug_force("NO_SUCH_SWITCH", 1)
    assert ei.value.status == 1
    B.apnn_debug_reset()


def test_tile_choice_follows_parallelism_first_then_compute_intensity():
    """Sec. 4.3: the most parallel candidate when even it cannot fill the chip, else the largest tile (highest compute
    intensity, Eq. 4) whose block count (Eq. 3) still reaches its threshold.  Host only: nothing is launched."""
    B.apnn_debug_reset()
    pick = B.apnn_debug_tile_choice
    for dim in range(128, 1025, 128):                                  # the paper's fully connected shapes, batch 64
        assert pick(dim, 64) == 32 and pick(dim, 64, matrix_form=False) == 32
    assert pick(4096, 4096) == 256 and pick(2048, 2048) == 128 and pick(4096, 4096, matrix_form=False) == 64
    assert pick(1024, 1024, matrix_form=False) == 64 and pick(1000, 1000, matrix_form=False) == 64   # 256 blocks of 64
    assert pick(1000, 900, matrix_form=False) == 32                    # 240 blocks of 64: parallelism first
    assert pick(3072, 3072) == 128 and pick(3584, 3584) == 256         # 144 / 196 blocks of 256: threshold 192
    assert pick(2048, 1024) == 32 and pick(100000, 70) == 64           # 512 blocks of 64: below 1024; 128-wide tiles 45 % empty
    assert pick(4096, 1024) == 128                                     # 256 blocks of 128
    assert pick(200000, 100) == 128                                    # ragged N: a 256-wide tile would be 61 % empty
    prev = 0
    for n in (64, 256, 1024, 2048, 4096, 8192):                        # never a smaller tile for a larger square
        t = pick(n, n)
        assert t >= prev
        prev = t
    assert pick(25088, 64, is_conv=True) == 32                         # convolutions: the lane-private kernel
    B.apnn_debug_force("MFMA_TILE", 64)
    assert pick(4096, 4096) == 64
    B.apnn_debug_reset()
    assert pick(0, 5) == 0


def test_sizes():
    assert B.apnn_row_words(1) == 4 and B.apnn_row_words(128) == 4 and B.apnn_row_words(129) == 8
    assert B.apnn_row_words(4096) == 128 and B.apnn_row_words(0) == 0
    assert B.apnn_packed_words(4096, 4096, 2) == 4096 * 2 * 128
    assert B.apnn_packed_words(3, 100, 9) == 0
    assert B.apnn_fmap_words(6272, 128, 2) == 6272 * 2 * 4
    assert B.apnn_fmap_words(10, 33, 1) == 20


def _status(fn, *args):
    rc = fn(*args)
    return rc, B.lib().apnn_last_error().decode()


def test_gemm_argument_validation():
    L = B.lib()
    ok = (FAKE, FAKE, FAKE, 8, 8, 64, 1, 2, B.ENC_PM1, B.ENC_UNSIGNED, None)

    def call(**kw):
        a = list(ok)
        names = ["W", "X", "Y", "M", "N", "K", "p", "q", "encW", "encX", "stream"]
        for k, v in kw.items():
            a[names.index(k)] = v
        return _status(L.apnn_gemm, *a)

    assert call(p=0)[0] == 2 and call(q=9)[0] == 2
    assert call(p=2)[0] == 2                           # +-1 with two bits
    assert call(encW=7)[0] == 1
    assert call(M=-1)[0] == 1
    assert call(Y=None)[0] == 1 and call(W=None)[0] == 1
    assert call(W=FAKE + 4)[0] == 4                    # misaligned packed operand
    rc, msg = call(K=40000, p=8, q=8, encW=B.ENC_UNSIGNED)
    assert rc == 3 and "int32" in msg                  # 40000 * 255 * 255 >= 2^31
    assert call(M=0)[0] == 0 and call(N=0)[0] == 0     # empty problems succeed without a launch


def test_pack_and_quantize_validation():
    L = B.lib()
    assert _status(L.apnn_pack, FAKE, 4, 64, 0, 0, FAKE, None)[0] == 2
    assert _status(L.apnn_pack, FAKE, 4, 64, 2, B.ENC_PM1, FAKE, None)[0] == 2
    assert _status(L.apnn_pack, None, 4, 64, 2, 0, FAKE, None)[0] == 1
    assert _status(L.apnn_pack, FAKE, 4, 64, 2, 0, FAKE + 8, None)[0] == 4
    assert _status(L.apnn_pack, FAKE, 0, 64, 2, 0, FAKE, None)[0] == 0
    assert _status(L.apnn_quantize, FAKE, 4, 64, 0.0, 0.0, 2, FAKE, None)[0] == 1     # step must be > 0
    assert _status(L.apnn_pack_patches, FAKE, 1, 3, 8, 8, 7, 12, 2, 3, 8, FAKE, None)[0] == 2   # 12*3 bits > 32
    assert _status(L.apnn_pack_fmap, FAKE, 5, 1, 4, 4, 32, 2, 0, FAKE, None)[0] == 1
    assert _status(L.apnn_sumpool, FAKE, 1, 7, 7, 64, 2, 7, FAKE, None)[0] == 3          # 147 needs 8 bits
    assert _status(L.apnn_maxpool, FAKE, 1, 8, 8, 64, 2, 3, 2, 3, FAKE, None)[0] == 1    # pad >= window


def test_layer_validation():
    L = B.lib()
    d = B.Conv(8, 28, 28, 128, 128, 3, 3, 1, 1)

    def layer(conv=d, **kw):
        args = dict(is_gemm=0, q_out=2, scale=FAKE, bias=FAKE, res=None, q_res=0, rs=0.0, acc=None, fo=None,
                    W=FAKE, X=FAKE, out=FAKE, pool=0)
        args.update(kw)
        desc = B.LayerDesc(conv.c(), args["is_gemm"], args["q_out"], args["scale"], args["bias"], args["res"],
                           args["q_res"], args["rs"], args["acc"], args["fo"], args["pool"])
        return _status(L.apnn_layer, C.byref(desc), args["W"], args["X"], args["out"], None)

    assert layer(conv=B.Conv(8, 28, 28, 100, 128, 3, 3, 1, 1))[0] == 1      # Cin not a multiple of 32
    assert layer(conv=B.Conv(8, 28, 28, 128, 100, 3, 3, 1, 1))[0] == 1      # packed output needs Cout % 32 == 0
    assert layer(scale=None)[0] == 1
    assert layer(out=None)[0] == 1
    assert layer(q_out=0)[0] == 1                                           # nothing requested
    assert layer(q_out=9)[0] == 2
    assert layer(res=FAKE, q_res=0)[0] == 2
    assert layer(pool=3)[0] == 1                                            # not an apnn_pool value
    assert layer(conv=B.Conv(8, 1, 1, 128, 128, 1, 1, 1, 0), is_gemm=1, pool=1)[0] == 1
    assert layer(conv=B.Conv(8, 2, 2, 128, 128, 7, 7, 1, 1))[0] == 1        # kernel larger than padded frame
    assert layer(is_gemm=1)[0] == 1                                         # gemm layer with H = 28
    assert layer(conv=B.Conv(0, 28, 28, 128, 128, 3, 3, 1, 1))[0] == 0      # empty batch
    assert _status(L.apnn_conv2d, None, FAKE, FAKE, FAKE, None)[0] == 1
    assert _status(L.apnn_layer_pair, None, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None)[0] == 1
    assert _status(L.apnn_input_layer, None, FAKE, FAKE, FAKE, None)[0] == 1


def test_fold_bn_matches_oracle_fold():
    rng = np.random.default_rng(0)
    g, b, m = rng.normal(1, .2, 64), rng.normal(0, 1, 64), rng.normal(0, 10, 64)
    v = rng.uniform(1, 50, 64)
    s1, b1 = B.apnn_fold_bn(g, b, m, v, 1e-5, 0.25, 0.5)
    s2, b2 = oracle.fold_bn(g, b, m, v, 1e-5, 0.25, 0.5)
    assert np.array_equal(s1, s2) and np.array_equal(b1, b2)
    with pytest.raises(B.ApnnError):
        B.apnn_fold_bn(g, b, m, v, 1e-5, 0.0, 0.0)
