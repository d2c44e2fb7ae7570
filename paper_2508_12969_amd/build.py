"""Builds libcompact_attn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
LIB_PATH = os.path.join(PKG_DIR, "libcompact_attn.so")
SOURCES = ["layout.cpp", "search.cpp", "api.cpp", "permute.hip", "attn_f32.hip", "attn_bf16.hip", "attn_bf16_pair.hip",
           "tile_mass.hip"]
PER_FILE_FLAGS = {}   # extra hipcc flags for single sources, if any
ARCH = "gfx950"


def hipcc_path():
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose=False, extra_flags=(), out=None):
    """Compile every source for gfx950 and link the shared library. Always recompiles."""
    common = [
        hipcc_path(), "-x", "hip", f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 VALU forms
        "-Wno-unused-command-line-argument",
        "-I", INCLUDE, "-I", CSRC,
        *extra_flags,
    ]
    obj_dir = os.path.join(os.path.dirname(out or LIB_PATH), "_build")
    os.makedirs(obj_dir, exist_ok=True)
    noise = "packed-fp32-ops"

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed:\n{err}")
        if verbose and err.strip():
            print(err)

    objs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src + ".o")
        run(common + PER_FILE_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    run([hipcc_path(), f"--offload-arch={ARCH}", "-shared", "-fPIC", *objs, "-o", out or LIB_PATH])
    return out or LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
