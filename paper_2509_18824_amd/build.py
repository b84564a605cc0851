"""Builds libhb.so (the C-ABI library) from csrc/*.hip with hipcc for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libhb.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Per-file code generation options.  The attention kernel reads every MFMA result (the scores)
# with vector instructions and keeps its accumulators in place anyway: with the matrix
# instructions selected in their vector-register form there are no accumulation registers and
# no copies between the two register files.
FILE_FLAGS = {
    "attn_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str, verbose: bool) -> str:
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless, filtered
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    return obj


def build(verbose: bool = False, jobs: int = 8) -> str:
    os.makedirs(BUILD, exist_ok=True)
    srcs = sources()
    with ThreadPoolExecutor(max_workers=min(jobs, len(srcs))) as ex:
        objs = list(ex.map(lambda s: _compile(s, verbose), srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB


def build_host_sanitizer_check(driver_c: str) -> str:
    """Builds a host program from `driver_c` and the library's objects, with the host code of
    csrc/hb_api.hip (validation, planning, error text) compiled under AddressSanitizer and
    UndefinedBehaviorSanitizer (device code is not instrumented).  Returns the executable."""
    out_dir = os.path.join(BUILD, "san")
    os.makedirs(out_dir, exist_ok=True)
    others = [os.path.join(BUILD, s.replace(".hip", ".o")) for s in sources() if s != "hb_api.hip"]
    if not all(os.path.exists(o) for o in others):
        build()
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer"]
    api_o = os.path.join(out_dir, "hb_api.o")
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g"]
    host_san = [x for f in san for x in ("-Xarch_host", f)]
    drv_o = os.path.join(out_dir, "driver.o")
    exe = os.path.join(out_dir, "host_sanitize_check")
    clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    for cmd in (
        [HIPCC, *flags, *host_san, "-c", os.path.join(CSRC, "hb_api.hip"), "-o", api_o],
        [clang, *san, "-g", "-I", os.path.join(ROOT, "include"), "-c", driver_c, "-o", drv_o],
        [HIPCC, "--offload-arch=gfx950", "-fno-gpu-rdc", *san, "-fno-gpu-sanitize", drv_o, api_o, *others, "-o", exe],
    ):
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"sanitizer build failed: {' '.join(cmd)}\n{r.stderr}")
    return exe


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
