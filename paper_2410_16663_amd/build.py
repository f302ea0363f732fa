"""Build the C-ABI HIP library (csrc/fa_fwd.hip -> libfa.so) for gfx950 with hipcc, and the host-side
library of the CPU-GPU cooperative strategy (csrc/fa_cpu.c -> libfa_cpu.so) with gcc.

hipcc cross-compiles without a GPU, so this runs on any machine with ROCm installed.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "fa_fwd.hip")
HDR = os.path.join(os.path.dirname(HERE), "include", "fa.h")
# fragments of the one translation unit, included by fa_fwd.hip
FRAGMENTS = [os.path.join(HERE, "csrc", n) for n in (
    "fa_types.inc", "fa_mask.inc", "fa_device.inc", "fa_attention_kernel.inc", "fa_attention_wide64_kernel.inc",
    "fa_linear_kernel.inc", "fa_decode_kernels.inc", "gen_fa_wide64_loop.py")]
# written by gen_fa_wide64_loop.py at build time (hand-scheduled assembly of a regular loop: generated, not typed)
GENERATED = os.path.join(HERE, "csrc", "fa_attention_wide64_loop.inc")
LIB = os.path.join(HERE, "libfa.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++20", "-shared", "-fPIC",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
    # per-kernel register / scratch / LDS report on stderr, checked below
    "-Rpass-analysis=kernel-resource-usage",
]

# kernel name -> {"VGPRs": n, "ScratchSize [bytes/lane]": n, ...} of the last build
last_report: dict = {}


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in [SRC, HDR] + FRAGMENTS)


def generate_fragments() -> None:
    """Run the generator of the wide64 kernel's main loop (the compile includes its output)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("gen_fa_wide64_loop", os.path.join(HERE, "csrc", "gen_fa_wide64_loop.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.generate(GENERATED)


def parse_resource_report(stderr: str) -> dict:
    """Collect the compiler's kernel-resource-usage remarks into {kernel: {field: int}}."""
    import re
    report, cur = {}, None
    for line in stderr.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            cur = report.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z][A-Za-z \[\]/]*?): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return report


def check_resource_report(report: dict) -> None:
    """The kernels are written to run from registers alone: any scratch memory (a spill, or a
    lambda the compiler left as a real call) is a performance bug of a factor of tens."""
    if not report:
        raise RuntimeError("no kernel-resource-usage remarks found: cannot check the build")
    for name, r in report.items():
        bad = {k: v for k, v in r.items() if k in ("ScratchSize [bytes/lane]", "VGPRs Spill") and v}
        if bad:
            raise RuntimeError(f"kernel {name} uses scratch memory: {bad}")
        if "fa_fwd_wide64_kernel" in name:
            continue        # one wave per SIMD by design: the whole register file
        if r.get("VGPRs", 0) + r.get("AGPRs", 0) > 256:
            raise RuntimeError(f"kernel {name} needs more than 256 registers: two waves per SIMD no longer fit")


def build(force: bool = True, verbose: bool = False, extra=()) -> str:
    """Compile libfa.so. ``force=False`` skips the compile when the library is newer than its sources."""
    if not force and not is_stale():
        return LIB
    generate_fragments()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + [SRC, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature and says so: harmless
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{r.stdout}\n{r.stderr}")
    global last_report
    last_report = parse_resource_report(r.stderr)
    check_resource_report(last_report)
    if verbose:
        for name, rep in last_report.items():
            print(f"{name}: VGPRs {rep.get('VGPRs')} LDS {rep.get('LDS Size [bytes/block]')}", file=sys.stderr)
    return LIB


CPU_SRC = os.path.join(HERE, "csrc", "fa_cpu.c")
CPU_HDR = os.path.join(os.path.dirname(HERE), "include", "fa_cpu.h")
CPU_LIB = os.path.join(HERE, "libfa_cpu.so")


def build_cpu(force: bool = True) -> str:
    """Compile libfa_cpu.so (plain C + OpenMP; the AVX-512 loops are compiled for that target inside the file
    and chosen at run time, so no -march flag here)."""
    if not force and os.path.exists(CPU_LIB) and all(
            os.path.getmtime(f) <= os.path.getmtime(CPU_LIB) for f in (CPU_SRC, CPU_HDR)):
        return CPU_LIB
    cmd = [os.environ.get("CC", "gcc"), "-O3", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", CPU_SRC, "-o",
           CPU_LIB, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gcc failed:\n{r.stdout}\n{r.stderr}")
    return CPU_LIB


BENCH_SRC = os.path.join(HERE, "csrc", "fa_bench.hip")
BENCH_LIB = os.path.join(HERE, "libfa_bench.so")
BENCH_CPU_SRC = os.path.join(HERE, "csrc", "fa_bench_cpu.c")
BENCH_CPU_LIB = os.path.join(HERE, "libfa_bench_cpu.so")


def build_bench(force: bool = True):
    """Compile the benchmark's measurement aids (include/fa_bench.h): libfa_bench.so with hipcc (the matrix-only
    probe kernel) and libfa_bench_cpu.so with gcc (the host streaming-read yardstick)."""
    out = []
    for src, lib, cmd in (
            (BENCH_SRC, BENCH_LIB, [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")]
             + [f for f in HIPCC_FLAGS if not f.startswith("-Rpass")]),
            (BENCH_CPU_SRC, BENCH_CPU_LIB, [os.environ.get("CC", "gcc"), "-O3", "-fopenmp", "-shared", "-fPIC", "-Wall",
                                            "-Wextra"])):
        if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
            r = subprocess.run(cmd + [src, "-o", lib], capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(f"building {lib} failed:\n{r.stdout}\n{r.stderr}")
        out.append(lib)
    return out


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    print(build_cpu(force=True))
    print(build_bench(force=True))
