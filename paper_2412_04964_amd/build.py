"""Compile the HIP sources for gfx950 into ``libfc.so`` next to this file.

    python -m paper_2412_04964_amd.build

hipcc cross-compiles without a GPU.  Flags that matter for bit-parity with the
arithmetic contract in include/fc.h:
  -ffp-contract=off          no implicit fused multiply-add (fmaf is explicit)
  no fast-math, IEEE divide  hipcc defaults, left alone
  packed-fp32 ops disabled   the build never emits v_pk_*_f32
and one that matters for speed:
  -amdgpu-kernarg-preload-count=16   the leading kernel arguments arrive in scalar registers when a
                             wavefront starts instead of being read from memory first (gfx940 and
                             later); the kernels' wavefronts live for one tile, so the saved read
                             is 1 % of the fused kernel's time
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfc.so")
BENCH_LIB = os.path.join(HERE, "libfc_bench.so")      # measurement aid (include/fc_bench.h), not the product
# the product library with the kernels that use landing zones (the fused kernels, the one-launch all-reduce) compiled
# with -DFC_PLAIN_LANDING_READS (plain, compiler-ordered reads of the landing zones instead of the hand-ordered
# ones): the GPU tests run those cases through both
PLAIN_LIB = os.path.join(HERE, "libfc_plainreads.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"
FLAGS = [
    "--offload-arch=" + ARCH, "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    "-I", INCLUDE, "-I", CSRC,
]

# (source, object suffix, extra defines)
UNITS = [("fc_api.hip", "api", []), ("fc_codec.hip", "codec", []), ("fc_wide.hip", "wide", []),
         ("fc_rot.hip", "rot", []), ("fc_small.hip", "small", [])]
for _c in range(4):      # one unit per quantizer: asymmetric, symmetric, FP8, asymmetric with binary16 metadata
    UNITS.append(("fc_sim.hip", "sim_%d" % _c, ["-DFC_SIM_CODEC=%d" % _c]))
BENCH_UNITS = [("fc_bench.hip", "bench", [])]
for _bi in (4, 8):
    for _bo in (4, 8):
        UNITS.append(("fc_fused.hip", "fused_%d_%d" % (_bi, _bo),
                      ["-DFC_BITS_IN=%d" % _bi, "-DFC_BITS_OUT=%d" % _bo]))


LANDING_SOURCES = ("fc_fused.hip", "fc_sim.hip")
PLAIN_UNITS = [(src, tag + "_plain", defs + ["-DFC_PLAIN_LANDING_READS"]) for src, tag, defs in UNITS
               if src in LANDING_SOURCES]


def _compile(unit):
    src, tag, defs = unit
    obj = os.path.join(OBJDIR, tag + ".o")
    cmd = [HIPCC, *FLAGS, *defs, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (tag, " ".join(cmd), r.stderr))
    warn = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    return obj, "\n".join(warn)


def build(verbose: bool = False, jobs: int | None = None) -> str:
    """Compile every unit (always; this is the "does it build" check) and link."""
    os.makedirs(OBJDIR, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(jobs) as ex:
        results = list(ex.map(_compile, UNITS + BENCH_UNITS + PLAIN_UNITS))
    if verbose:
        for _, w in results:
            if w:
                print(w, file=sys.stderr)
    objs = [o for o, _ in results]
    n_u, n_b = len(UNITS), len(BENCH_UNITS)
    shared = [o for o, (src, _, _) in zip(objs[:n_u], UNITS) if src not in LANDING_SOURCES]
    for lib, members in ((LIB, objs[:n_u]), (BENCH_LIB, objs[n_u:n_u + n_b]), (PLAIN_LIB, shared + objs[n_u + n_b:])):
        tmp = lib + ".tmp.%d" % os.getpid()
        cmd = [HIPCC, "--offload-arch=" + ARCH, "-shared", "-fPIC", "-o", tmp, *members]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s" % r.stderr)
        os.replace(tmp, lib)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
