"""Build libsbgemm.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libsbgemm.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

SOURCES = ["sb_api.cpp", "mapper.cpp", "kernels_generic.hip", "kernels_tiny.hip", "kernels_thin.hip", "kernels_mfma.hip", "kernels_mfma_bf16.hip", "kernels_panel_bf16.hip", "kernels_mfma_ex.hip", "kernels_eig.hip", "kernels_probe.hip", "kernels_permute.hip", "tucker.cpp"]

# -packed-fp32-ops is switched off on purpose: the compiler must not form packed fp32 arithmetic.
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument"]


def _compile(src: str, verbose: bool) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if src.endswith(".hip"):
        cmd = [HIPCC] + COMMON + DEVICE_FLAGS + ["-c", path, "-o", obj]
    else:
        cmd = [HIPCC] + COMMON + ["-x", "hip", "--offload-arch=gfx950", "-c", path, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return obj


def _stale(src: str) -> bool:
    """True if the object of `src` is missing or older than the source or any header."""
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    if not os.path.exists(obj):
        return True
    deps = [os.path.join(CSRC, src)] + [os.path.join(CSRC, h) for h in os.listdir(CSRC) if h.endswith(".h")]
    inc = os.path.join(os.path.dirname(PKG), "include")
    deps += [os.path.join(inc, h) for h in os.listdir(inc)]
    return any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps)


def build(verbose: bool = False, only_changed: bool = False) -> str:
    """Compile every source and link libsbgemm.so; returns its path.  Recompiles everything unless
    only_changed is set (a developer's shortcut: sources newer than their objects, or all of them
    after a header changed)."""
    os.makedirs(OBJ, exist_ok=True)
    todo = [s for s in SOURCES if not only_changed or _stale(s)]
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        list(pool.map(lambda s: _compile(s, verbose), todo))
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, only_changed="--changed" in sys.argv))
