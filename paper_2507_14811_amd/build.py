"""Builds libsegquant.so (HIP, gfx950 only) in-tree with hipcc.

Every source is compiled to an object in parallel (the MFMA kernel once per tile variant, each in a
translation unit of its own) and linked into ``paper_2507_14811_amd/libsegquant.so``; the benchmark probes
(``csrc/probes.hip``) become ``libsegquant_probes.so``.
Run as ``python -m paper_2507_14811_amd.build``.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libsegquant.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # packed fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unknown-warning-option", "-Wno-unused-command-line-argument",
    f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}",
]
PLAIN_SOURCES = ["api.hip", "quantize.hip", "seglinear_generic.hip", "seglinear_skinny.hip", "seglinear_stream.hip", "calibrate.hip",
                 "seglinear_mfma.hip", "smooth.hip", "lowrank.hip", "fp8.hip"]
# benchmark probes: a library of their own (include/segquant_probes.h), loaded by bench.py only
PROBE_LIB = os.path.join(PKG, "libsegquant_probes.so")


def _num_variants() -> int:
    with open(os.path.join(CSRC, "seglinear_mfma_variants.hpp")) as f:
        return int(re.search(r"kNumMfmaVariants\s*=\s*(\d+)", f.read()).group(1))


def _fp8_variants() -> list:
    with open(os.path.join(CSRC, "seglinear_mfma_variants.hpp")) as f:
        flags = re.search(r"kMfmaVariantHasFp8\[[^\]]*\]\s*=\s*\{([^}]*)\}", f.read()).group(1)
    return [i for i, t in enumerate(flags.split(",")) if t.strip() == "true"]


def _jobs():
    jobs = [(os.path.join(CSRC, s), os.path.join(OBJ, s.replace(".hip", ".o")), []) for s in PLAIN_SOURCES]
    for v in range(_num_variants()):
        jobs.append((os.path.join(CSRC, "seglinear_mfma_inst.hip"), os.path.join(OBJ, f"seglinear_mfma_v{v}.o"),
                     [f"-DSQ_VARIANT={v}"]))
    # the weight-stream kernel on fp8 codes: the same source, a translation unit of its own
    jobs.append((os.path.join(CSRC, "seglinear_stream.hip"), os.path.join(OBJ, "seglinear_stream_fp8.o"), ["-DSQ_STREAM_FP8=1"]))
    for v in _fp8_variants():          # the same tiles on fp8 codes
        jobs.append((os.path.join(CSRC, "seglinear_mfma_inst.hip"), os.path.join(OBJ, f"seglinear_mfma_fp8_v{v}.o"),
                     [f"-DSQ_VARIANT={v}", "-DSQ_FP8=1"]))
    return jobs


def _compile(job):
    src, obj, extra = job
    cmd = [HIPCC, *FLAGS, *extra, *os.environ.get("SQ_EXTRA_HIPCC_FLAGS", "").split(), "-c", src, "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {os.path.basename(obj)}:\n{out}")
    return out


def build_library(verbose: bool = True, jobs: int | None = None) -> str:
    """Compile every HIP source for gfx950 and link the shared library.  Returns its path."""
    os.makedirs(OBJ, exist_ok=True)
    todo = _jobs()
    workers = jobs or min(8, os.cpu_count() or 4)
    with ThreadPoolExecutor(max_workers=workers) as ex:
        for job, out in zip(todo, ex.map(_compile, todo)):
            if verbose:
                print(f"[build] {os.path.basename(job[1])}", flush=True)
                if out:
                    print(out, flush=True)
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *[j[1] for j in todo]]
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    if verbose:
        print(f"[build] linked {LIB}", flush=True)
    tmp = PROBE_LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, *FLAGS, "-shared", os.path.join(CSRC, "probes.hip"), "-o", tmp]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for the probe library:\n" + r.stdout)
    os.replace(tmp, PROBE_LIB)
    if verbose:
        print(f"[build] linked {PROBE_LIB}", flush=True)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
