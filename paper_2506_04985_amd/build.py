"""Compile the HIP sources under csrc/ for gfx950 into csrc/libfptq.so, and the measurement aids into
csrc/libfptq_probe.so (in-tree, so that the built libraries travel with the source tree)."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(CSRC, "libfptq.so")
PROBE_LIB = os.path.join(CSRC, "libfptq_probe.so")
SOURCES = ["fptq_api.hip", "fptq_pack.hip", "fptq_quant.hip", "fptq_gemm.hip", "fptq_gemv.hip", "fptq_hadamard.hip", "fptq_residual.hip"]
PROBE_SOURCES = ["fptq_probe.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-I", INCLUDE, "-I", CSRC]


def _compile(src):
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    p = subprocess.run([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    return obj, out


def build(verbose: bool = False) -> str:
    with ThreadPoolExecutor(max_workers=len(SOURCES) + len(PROBE_SOURCES)) as ex:
        results = list(ex.map(_compile, SOURCES + PROBE_SOURCES))
    if verbose:
        for _, out in results:
            if out.strip():
                print(out)
    objs = [o for o, _ in results]
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs[:len(SOURCES)], "-o", LIB])
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs[len(SOURCES):], "-o", PROBE_LIB])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
