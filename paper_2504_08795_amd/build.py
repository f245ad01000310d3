"""Builds libdaris.so for gfx950 with hipcc, in-tree: the device code object (every kernel of csrc/kernels.hip), linked
into the library as data, and the host runtime that dispatches it (HSA queues) behind the C ABI."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdaris.so")
CODE_OBJECT = os.path.join(CSRC, "daris_kernels.co")
HOST_SOURCES = ["aql.cpp", "launch.cpp", "sched_core.cpp", "net_plan.cpp", "daris_api.cpp"]
COMMON = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function"]
# no packed fp32 arithmetic in device code (some forms have given wrong results on this hardware)
DEVICE_FLAGS = COMMON + ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "--cuda-device-only", "--no-gpu-bundle-output"]
HOST_FLAGS = COMMON + ["-fPIC"]

BLOB_ASM = """
    .section .rodata
    .global daris_kernels_co
    .global daris_kernels_co_end
    .balign 4096
daris_kernels_co:
    .incbin "{path}"
daris_kernels_co_end:
    .byte 0
    .section .note.GNU-stack,"",@progbits
"""


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc] + DEVICE_FLAGS + ["-c", os.path.join(CSRC, "kernels.hip"), "-o", CODE_OBJECT], verbose)
    blob_s = os.path.join(CSRC, "kernels_blob.S.tmp.s")
    with open(blob_s, "w") as f:
        f.write(BLOB_ASM.format(path=CODE_OBJECT))
    objs = [os.path.join(CSRC, "kernels_blob.o")]
    _run(["gcc", "-c", blob_s, "-o", objs[0]], verbose)
    os.remove(blob_s)
    # the one translation unit with both host and device code: the static scratch array and its address lookup
    obj = os.path.join(CSRC, "static_scratch.hip.o")
    _run([hipcc] + HOST_FLAGS + ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-c", os.path.join(CSRC, "static_scratch.hip"), "-o", obj], verbose)
    objs.append(obj)
    for src in HOST_SOURCES:
        obj = os.path.join(CSRC, src + ".o")
        _run([hipcc] + HOST_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj], verbose)
        objs.append(obj)
    _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs + ["-L/opt/rocm/lib", "-lhsa-runtime64", "-lpthread", "-ldl"], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
