"""Build libaq.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libaq.so")
SOURCES = ["aq_api.hip", "aq_api_cb.hip", "aq_pack.hip", "aq_gemv.hip", "aq_gemv_cb.hip", "aq_gemv2.hip", "aq_gemm.hip", "aq_gemm2.hip", "aq_gemm_small.hip", "aq_gemm_pc.hip", "aq_gemm_pcx.hip", "aq_quant.hip",
           "aq_layer.hip", "aq_hsic.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Wall", "-Wno-unused-result",
    # packed-fp32 VALU forms are kept out of the generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
# per-source additions
SOURCE_FLAGS = {
    # prefill: MFMA results in ordinary VGPRs (no AGPR copies around the fp32 scaling of block sums).
    # Only here: the decode kernel is 8% slower with it.
    "aq_gemm.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "aq_gemm2.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
}


def _run(cmd: list[str], verbose: bool) -> str:
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    text = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + text)
    return text


def build(verbose: bool = False, extra: list[str] | None = None, out: str | None = None) -> str:
    """Compile every source to an object of its own (in a temporary folder), then link the shared library."""
    import concurrent.futures
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = out or LIB
    log = []
    with tempfile.TemporaryDirectory(prefix="aq_build_") as tmp:
        jobs = []
        for src in SOURCES:
            obj = os.path.join(tmp, src.replace(".hip", ".o"))
            jobs.append((obj, [hipcc] + HIPCC_FLAGS + SOURCE_FLAGS.get(src, []) + (extra or []) +
                         ["-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj]))
        with concurrent.futures.ThreadPoolExecutor(max_workers=6) as pool:
            log += list(pool.map(lambda j: _run(j[1], verbose), jobs))
        log.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + [j[0] for j in jobs], verbose))
    text = "\n".join(t for t in log if t.strip())
    if verbose and text:
        print(text)
    return text


def build_extra(src: str, out: str, verbose: bool = False) -> str:
    """One-file shared library with the same flags (the bench's calibration probe lives outside the package)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return _run([hipcc] + HIPCC_FLAGS + ["-shared", "-o", out, src], verbose)


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
