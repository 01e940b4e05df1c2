"""Compile the HIP library for gfx950 into paper_2006_11735_amd/libicnn_mi355.so."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libicnn_mi355.so")
SOURCES = ["api.hip", "conv_igemm.hip", "conv_dual.hip", "conv_halo.hip", "conv_deep.hip", "conv_plane.hip", "conv_block.hip", "conv_block64.hip", "conv_pair.hip", "conv_stem.hip", "conv_pic.hip", "conv_fc.hip", "conv_narrow.hip", "eltwise.hip", "peaks.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose=False, extra=(), only_changed=False):
    """only_changed: skip sources whose object is newer than the source and every header (development aid;
    the driver's build check compiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(HERE, "..", "include", "icnn.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)

    def compile_one(src):
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        if only_changed and os.path.exists(obj) and os.path.getmtime(obj) > max(newest_header,
                                                                                os.path.getmtime(os.path.join(CSRC, src))):
            return obj
        cmd = [hipcc] + FLAGS + list(extra) + ["-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=10) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, only_changed="--changed" in sys.argv))
