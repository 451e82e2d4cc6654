"""Compile the HIP sources of the LAQ library for gfx950 into an in-tree shared object."""
from __future__ import annotations

import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "liblaq.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # let MFMA results land in ordinary VGPRs: the softmax consumes them directly
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(f) > t for f in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Run hipcc (cross-compiles without a GPU): every source to an object file, side by side, then one
    link.  Returns the path of the library."""
    if not force and not needs_build():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    include = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]

    def run(cmd):
        res = subprocess.run(cmd, capture_output=True, text=True)
        if verbose or res.returncode != 0:
            print(res.stdout)
            print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
        if res.returncode != 0:
            raise RuntimeError("hipcc failed (exit %d): %s" % (res.returncode, " ".join(cmd[-3:])))

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".%d.o" % os.getpid())
        run([hipcc] + compile_flags + include + ["-c", "-o", obj, src])
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as pool:
        objs = list(pool.map(compile_one, sources()))
    tmp = LIB + ".tmp.%d" % os.getpid()
    try:
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
