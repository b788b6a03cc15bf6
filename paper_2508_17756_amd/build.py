"""Builds libsupergen_tile.so (HIP kernels + C ABI) for gfx950, in tree, with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsupergen_tile.so")
PROBE = os.path.join(PKG, "peak_probe.bin")
C_CLIENT_SRC = os.path.join(ROOT, "tests", "c_client", "gpu_client.c")
C_CLIENT = os.path.join(ROOT, "tests", "c_client", "gpu_client.bin")
SOURCES = ["sg_api.hip", "attention_bf16.hip", "attention_bf16_generic.hip", "attention_f32.hip", "blend.hip",
           "gate.hip", "gate_static.hip", "region.hip", "similarity.hip"]
# per-file extras: the streaming attention kernel takes row maxima with three-operand max instructions,
# which the compiler only forms when it need not canonicalise NaNs
EXTRA = {"attention_bf16.hip": ["-fno-honor-nans"]}
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 VALU forms are kept out of the generated code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), err))
    return err


def build(verbose=False):
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        msg = _run([hipcc, *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj])
        if verbose and msg.strip():
            print(msg, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    # stand-alone probe of the device's achievable MFMA and HBM rates (bench.py sets it beside the vendor peaks)
    _run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          os.path.join(CSRC, "peak_probe.hip"), "-o", PROBE])
    # the plain C caller of the device-side entry points that the GPU tests start as a child process (host compiler only)
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    _run([os.environ.get("CC", "gcc"), "-std=c99", "-Wall", "-Wextra", "-O1", "-D__HIP_PLATFORM_AMD__",
          "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"), C_CLIENT_SRC, "-o", C_CLIENT,
          "-L", PKG, "-lsupergen_tile", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
          "-Wl,-rpath,$ORIGIN/../../paper_2508_17756_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
