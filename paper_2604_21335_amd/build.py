"""Builds libstc.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libstc.so")
BENCH_LIB_PATH = os.path.join(PKG_DIR, "libstc_bench.so")   # benchmark-only helpers (bench.py)
BUILD_DIR = os.path.join(PKG_DIR, "_build")

SOURCES = ["stc_api.hip", "bounds.hip", "router.hip", "route_pack.hip", "flush.hip",
           "score.hip", "select.hip", "attention.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # packed-FP32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
# matrix-core results are consumed by vector instructions right away, so keep them in
# ordinary vector registers (no copies out of the accumulation registers)
_VGPR_MFMA = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
FILE_FLAGS = {"score.hip": _VGPR_MFMA, "attention.hip": _VGPR_MFMA, "router.hip": _VGPR_MFMA}


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), r.stdout))
    return r.stdout


def build_library(verbose=False):
    """Compile every source and link libstc.so; always recompiles."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    hipcc = _hipcc()
    objs = [os.path.join(BUILD_DIR, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        out = _run([hipcc, *HIPCC_FLAGS, *FILE_FLAGS.get(src, []), "-c",
                    os.path.join(CSRC, src), "-o", obj])
        if verbose and out.strip():
            print(out)

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        list(ex.map(one, zip(SOURCES, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs])
    _run([hipcc, *HIPCC_FLAGS, "-shared", "-o", BENCH_LIB_PATH,
          os.path.join(CSRC, "bench_stream.hip")])
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
