"""Builds libla2.so (the C-ABI library) and libla2_bench.so (the benchmark's measurement kernels) for gfx950 with
hipcc, in-tree."""
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libla2.so")
SOURCES = ["la2_api.hip", "la2_scan_bf16.hip", "la2_scan_bf16_half.hip", "la2_chunk_state_bf16.hip",
           "la2_left_product_bf16.hip", "la2_scan_f32.hip", "la2_decode.hip", "la2_recur.hip", "la2_norm.hip", "la2_tail_bf16.hip", "la2_scan_wide.hip"]
BENCH_LIB = os.path.join(_HERE, "libla2_bench.so")
BENCH_SOURCES = ["bench_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 code generation
    "-mllvm", "-amdgpu-mfma-vgpr-form",   # MFMA accumulators in VGPRs: VALU touches them without AGPR copies
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
]


def build(verbose=False):
    """Compiles every HIP source and links libla2.so and libla2_bench.so.  Always rebuilds."""
    objs = []
    procs = []
    bdir = os.path.join(_HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    for src in SOURCES + BENCH_SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    for lib, part in ((LIB, objs[:len(SOURCES)]), (BENCH_LIB, objs[len(SOURCES):])):
        tmp = lib + ".tmp%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + part)
        os.replace(tmp, lib)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
