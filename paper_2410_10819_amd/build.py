"""Build libduoattn.so (and the input-generator twin) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libduoattn.so")
SYNTH_LIB = os.path.join(HERE, "libduosynth.so")

SOURCES = ["duo_api.hip", "kernels_append.hip", "kernels_decode.hip", "kernels_decode_sk.hip", "kernels_prefill.hip"]
SYNTH_SOURCES = ["synth_fill.hip"]
# -amdgpu-mfma-vgpr-form: matrix-core accumulators in ordinary vector registers.  Left to itself the
# compiler parks them in the accumulation registers once a kernel is allowed more than 256 registers
# (the decode kernels, one workgroup per compute unit) and then copies them back and forth for every
# vector instruction that touches them: 72-84 copies per 32-key block, a fifth of the loop's instructions.
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(line for line in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in line)      # host pass does not know the GPU feature
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    if out.strip():
        print(out, file=sys.stderr)


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    present = SOURCES + SYNTH_SOURCES
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in present]

    def compile_one(pair):
        src, obj = pair
        _run([hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
        if verbose:
            print("compiled", src)

    with ThreadPoolExecutor(max_workers=min(8, len(present))) as pool:
        list(pool.map(compile_one, zip(present, objs)))
    n = len(SOURCES)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs[:n]])
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", SYNTH_LIB, *objs[n:]])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
