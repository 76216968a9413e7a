"""Builds libadakv.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
# (source, extra defines, object name): the matrix-core scoring kernels are by far the longest
# compile, so their instantiations are built as four translation units side by side
UNITS = [("score_mfma.hip", ["-DADAKV_MFMA_PART=%d" % part], "score_mfma_%d.o" % part) for part in (1, 2, 3, 4)]
UNITS += [(src, [], src.replace(".hip", ".o")) for src in
          ("api.hip", "score_generic.hip", "select.hip", "compact.hip", "decode.hip", "probe.hip")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-fp32 VALU forms are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA accumulators straight in VGPRs: no accvgpr moves in front of the softmax math
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         "-Wall", "-Wno-unused-function"]


def build(verbose: bool = False, extra_flags=(), jobs: int = 6) -> str:
    from concurrent.futures import ThreadPoolExecutor
    out_dir = os.path.join(HERE, "lib")
    obj_dir = os.path.join(out_dir, "obj")
    os.makedirs(obj_dir, exist_ok=True)
    out = os.path.join(out_dir, "libadakv.so")
    includes = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]

    def compile_one(unit):
        src, defines, obj = unit
        cmd = (["hipcc"] + FLAGS + list(extra_flags) + defines + includes
               + ["-c", os.path.join(HERE, "csrc", src), "-o", os.path.join(obj_dir, obj)])
        if verbose:
            print(" ".join(cmd))
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n" % src + r.stdout + r.stderr)
        return r.stderr

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        logs = list(pool.map(compile_one, UNITS))
    cmd = (["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"]
           + [os.path.join(obj_dir, obj) for _, _, obj in UNITS] + ["-o", out])
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed to link:\n" + r.stdout + r.stderr)
    if verbose:
        print("".join(logs) + r.stderr)
    return out


def build_abi_driver(verbose: bool = False) -> str:
    """tests/abi_driver: a plain C++ caller of the C ABI (hipMalloc, default stream, no Python),
    linked against the library built above; used by one GPU test."""
    src = os.path.join(ROOT, "tests", "abi_driver.cpp")
    out = os.path.join(ROOT, "tests", "abi_driver.bin")
    lib_dir = os.path.join(HERE, "lib")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "include"), src,
           "-L", lib_dir, "-ladakv", "-Wl,-rpath,$ORIGIN/../paper_2407_11550_amd/lib", "-o", out]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stdout + r.stderr)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
