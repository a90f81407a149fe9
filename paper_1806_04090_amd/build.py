"""Builds libatomo.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_1806_04090_amd.build`.

`--host-ubsan` builds libatomo_host_ubsan.so beside it instead: the same sources with the host code (argument checks,
planners, descriptor tables) instrumented by UndefinedBehaviorSanitizer, any finding fatal.  Device code is not
instrumented (no GPU sanitizer here).  `ATOMO_LIB=<path>` makes the binding load that file, so
`ATOMO_LIB=paper_1806_04090_amd/libatomo_host_ubsan.so python -m pytest tests -m gpu` runs the GPU suite on it."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libatomo.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["capi.hip", "svd.hip", "svd_eig.hip", "svd_thin.hip", "entrywise.hip", "decode.hip"]

# packed-fp32 instructions are switched off on purpose: the compiler would otherwise form them
# from ordinary float code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-result",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


LIB_UBSAN = os.path.join(HERE, "libatomo_host_ubsan.so")
UBSAN_FLAGS = ["-g", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def _ubsan_runtime_dir(hipcc: str) -> str:
    out = subprocess.check_output([hipcc, "--print-file-name=libclang_rt.ubsan_standalone-x86_64.so"], text=True).strip()
    if not os.path.isabs(out):                       # not on the default search path: look under the compiler's resource dir
        res = subprocess.check_output([hipcc, "-print-resource-dir"], text=True).strip()
        out = os.path.join(res, "lib", "linux", "libclang_rt.ubsan_standalone-x86_64.so")
    return os.path.dirname(out)


def build(verbose: bool = False, host_ubsan: bool = False) -> str:
    obj_dir = OBJ_DIR + ("_ubsan" if host_ubsan else "")
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = _hipcc()
    extra = UBSAN_FLAGS if host_ubsan else []

    def compile_one(src: str) -> str:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    lib = LIB_UBSAN if host_ubsan else LIB
    tmp = lib + ".tmp.%d" % os.getpid()
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    if host_ubsan:                                   # the shared sanitizer runtime, found through an rpath
        link += ["-fsanitize=undefined", "-shared-libsan", "-Wno-option-ignored", "-Wl,-rpath," + _ubsan_runtime_dir(hipcc)]
    subprocess.check_call(link)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, host_ubsan="--host-ubsan" in sys.argv))
