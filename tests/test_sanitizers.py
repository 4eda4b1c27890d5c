"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU code is sanitized, none runs):
the C oracle on exact-size heap buffers, and the host side of the C-ABI library -- argument checks, size helpers,
the batch-norm fold, the override table and the whole kernel dispatch, with stand-ins for the kernel launchers
(tests/sanitize/*.c*).  Each program aborts on the first finding."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2106_12169_amd", "csrc")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-3000:] + r.stderr[-3000:]
    return r.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", *SAN, "-static-libasan", "-fno-omit-frame-pointer",
          os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "oracle.c"),
          "-o", exe, "-lm"])
    assert "oracle sanitizer run ok" in _run([exe])


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_abi_host_side_under_sanitizers(tmp_path):
    # the sanitizer flags go to the host pass only (each directly after -Xarch_host)
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]
    common = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-ffp-contract=off"]
    units = [os.path.join(CSRC, n) for n in ("layer.hip", "pack.hip", "pool.hip", "input_layer.hip", "common.cpp")]
    units.append(os.path.join(ROOT, "tests", "sanitize", "abi_host_driver.cpp"))

    def compile_one(src):
        obj = str(tmp_path / (os.path.splitext(os.path.basename(src))[0] + ".o"))
        _run([*common, "-x", "hip", *host_san, "-c", src, "-o", obj])
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, units))
    exe = str(tmp_path / "abi_san")
    _run(["hipcc", "--offload-arch=gfx950", *SAN, *objs, "-o", exe])
    assert "abi host sanitizer run ok" in _run([exe])
