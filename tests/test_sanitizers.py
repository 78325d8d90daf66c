"""CPU sanitizer targets: the C oracles and the host side of the C ABI under AddressSanitizer and
UndefinedBehaviorSanitizer.  Both programs live in tests/sanitize/, are compiled here and run without a GPU: the
oracle driver calls every oracle function on exact-size heap buffers, the ABI driver calls the size queries, the plan
builders, the bit allocator and the argument checks of the launching entry points (none gets as far as a launch)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
PKG = os.path.join(ROOT, "paper_2605_24011_amd")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600, **kw)
    text = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    return res.returncode, text


def test_c_oracles_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    rc, out = _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-o", exe, os.path.join(SAN, "oracle_driver.c"),
                    os.path.join(ROOT, "oracle", "aq_oracle.c"), os.path.join(ROOT, "oracle", "aq_scale_oracle.c"), "-lm"])
    assert rc == 0, out
    rc, out = _run([exe])
    assert rc == 0 and out.strip().endswith("ok"), out


@pytest.mark.skipif(not (shutil.which(HIPCC) or os.path.exists(HIPCC)), reason="hipcc not found")
def test_host_side_of_the_abi_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = os.path.join(PKG, "libaq.so")
    if not os.path.exists(lib):
        from paper_2605_24011_amd import build
        build.build()
    exe = str(tmp_path / "abi_san")
    # host pass instrumented, device pass untouched; the launchers of the kernels come from the built library
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"), "-o", exe,
           os.path.join(SAN, "abi_host_driver.cpp"), os.path.join(PKG, "csrc", "aq_api.hip"),
           "-L", PKG, "-laq", "-Wl,-rpath," + PKG]
    rc, out = _run(cmd)
    assert rc == 0, out
    rc, out = _run([exe])
    assert rc == 0 and out.strip().endswith("ok"), out
