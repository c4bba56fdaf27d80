"""Compile liblpp.so (HIP, gfx950) in-tree with hipcc: one object per source, side by side, then a link."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblpp.so")
SOURCES = ["lpp_tree.hip", "lpp_verify.hip", "lpp_attention.hip", "lpp_knn.hip", "lpp_commit.hip", "lpp_probe.hip"]
FLAGS = ["-O3", "-ffp-contract=off", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes", "-Wno-unused-command-line-argument"]


def build_library(verbose: bool = True, extra_flags=(), lib_path: str = LIB) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    names = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    tag = os.path.splitext(os.path.basename(lib_path))[0]
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]

    def compile_one(name):
        obj = os.path.join(OBJ, f"{tag}_{os.path.splitext(name)[0]}.o")
        cmd = [hipcc] + FLAGS + list(extra_flags) + inc + ["-c", os.path.join(CSRC, name), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        return name, obj, r

    with ThreadPoolExecutor(max_workers=min(8, len(names))) as pool:
        done = list(pool.map(compile_one, names))
    objs = []
    for name, obj, r in done:
        # (hipcc's host pass says that it does not know the packed-fp32 feature: harmless, not shown)
        text = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if text.strip() and (verbose or r.returncode != 0):
            print(text, flush=True)
        if r.returncode != 0:
            raise subprocess.CalledProcessError(r.returncode, name)
        objs.append(obj)
    cmd = [hipcc, "--offload-arch=gfx950", "-fno-gpu-rdc", "-shared", "-fPIC"] + objs + ["-o", lib_path]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib_path


if __name__ == "__main__":
    build_library()
    print(LIB)
