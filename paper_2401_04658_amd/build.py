"""Builds libla2.so (the C-ABI library) and libla2_bench.so (the benchmark's measurement kernels) for gfx950 with
hipcc, in-tree."""
import json
import os
import re
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
    "-Rpass-analysis=kernel-resource-usage",   # registers, scratch, LDS of every kernel -> _build/kernel_resources.json
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
]


RESOURCES = os.path.join(_HERE, "_build", "kernel_resources.json")
_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|TotalSGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                     r"VGPRs Spill|SGPRs Spill|LDS Size \[bytes/block\]|Dynamic Stack):\s+(\S+)")


def _take_resource_remarks(out, resources):
    """Moves the compiler's per-kernel resource remarks of the device pass from `out` into `resources`
    ({mangled kernel name: {"VGPRs": .., "ScratchSize": .., "Occupancy": .., "LDS": .., ...}}); returns the rest."""
    rest, name, skip = [], None, 0
    for line in out.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" in line:
            m = _REMARK.search(line)
            if m:
                key, val = m.group(1).split(" [")[0].replace(" Size", "").replace(" ", "_"), m.group(2)
                if key == "Function_Name":
                    name = val
                    resources[name] = {}
                elif name is not None:
                    resources[name][key] = int(val) if val.isdigit() else val
            skip = 2   # the two source-excerpt lines that follow a remark's first line
            continue
        if skip and (line.lstrip().startswith("|") or re.match(r"\s*\d+ \|", line)):
            skip -= 1
            continue
        skip = 0
        rest.append(line)
    return "\n".join(rest)


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
    resources = {}
    for src, pr in procs:
        out, _ = pr.communicate()
        out = _take_resource_remarks(out, resources)
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    with open(os.path.join(bdir, "kernel_resources.json"), "w") as f:
        json.dump(resources, f, indent=1, sort_keys=True)
    for lib, part in ((LIB, objs[:len(SOURCES)]), (BENCH_LIB, objs[len(SOURCES):])):
        tmp = lib + ".tmp%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + part)
        os.replace(tmp, lib)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
