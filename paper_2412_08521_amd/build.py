"""Build the gfx950 HIP library in-tree: paper_2412_08521_amd/libems_hip.so.

hipcc cross-compiles without a GPU.  Usage:  python -m paper_2412_08521_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OBJ_DIR = os.path.join(_HERE, "_build")
LIB = os.path.join(_HERE, "libems_hip.so")
SOURCES = ["ems_api.hip", "score.hip", "select.hip", "merge.hip", "decode.hip", "stats.hip"]
HEADERS = ["ems_common.h", "ems_kernels.h", "ems_rows.h", os.path.join("..", "..", "include", "ems.h")]
# the benchmark's ceiling measurements: a library of their own, outside the product's interface
PROBE_DIR = os.path.join(_HERE, "bench_probe")
PROBE_LIB = os.path.join(_HERE, "libems_probe.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-FP32 instruction selection is switched off for device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         # the LDS-DMA inline assembly names M0 as clobbered, which clang flags as reserved
         "-Wno-inline-asm"] + os.environ.get("EMS_EXTRA_HIPCC_FLAGS", "").split()
# The score kernels read every accumulator element with the vector ALU: matrix results go to
# ordinary vector registers, never to the accumulation file (which the ALU cannot read).
FILE_FLAGS = {"score.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1", "-Rpass-analysis=kernel-resource-usage"]}
# Kernels that count their own vector-memory operations (s_waitcnt vmcnt(n) by hand around the
# LDS DMA): a register spill would add scratch loads/stores the count does not know about, so
# such a build is rejected instead of being allowed to run with a silent race.
NO_SCRATCH = {"score.hip": ("score_pass1", "score_pass2")}


def _check_no_scratch(src: str, remarks: str) -> None:
    """Parse the compiler's kernel-resource-usage remarks; raise if a guarded kernel spills."""
    guarded = NO_SCRATCH.get(src, ())
    name, seen = None, set()
    for line in remarks.splitlines():
        if "remark:" not in line:
            continue
        text = line.split("remark:", 1)[1].strip()
        if text.startswith("Function Name:"):
            name = text.split(":", 1)[1].split("[")[0].strip()
        elif name and any(g in name for g in guarded):
            # (a "VGPRs Spill" that costs no scratch went to the accumulation registers: moves, not memory)
            for key in ("ScratchSize [bytes/lane]:",):
                if text.startswith(key):
                    val = int(text[len(key):].split("[")[0].strip())
                    seen.add(name)
                    if val != 0:
                        raise RuntimeError(f"{src}: kernel {name} reports '{key} {val}'; the hand-counted "
                                           "s_waitcnt vmcnt() of its DMA pipeline requires zero scratch")
    if guarded and not seen:
        raise RuntimeError(f"{src}: no resource-usage remark found for kernels {guarded}")


def _stale(out: str, deps) -> bool:
    if not os.path.exists(out):
        return True
    t = os.path.getmtime(out)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdrs = [os.path.normpath(os.path.join(CSRC, h)) for h in HEADERS]

    def compile_one(src):
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        if force or _stale(o, [s] + hdrs):
            cmd = [HIPCC] + FLAGS + FILE_FLAGS.get(src, []) + ["-c", s, "-o", o]
            r = subprocess.run(cmd, capture_output=True, text=True)
            err = "\n".join(l for l in r.stderr.splitlines()
                            if "packed-fp32-ops' is not a recognized feature" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{err}")
            if src in NO_SCRATCH:
                try:
                    _check_no_scratch(src, err)
                except RuntimeError:
                    os.remove(o)          # never link an object that failed the check
                    raise
                err = "\n".join(l for l in err.splitlines() if "kernel-resource-usage" not in l
                                and not l.lstrip().startswith(("|", "^")) and "{" != l.strip()[-1:])
            if verbose and err.strip():
                print(err, file=sys.stderr)
        return o

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    if force or _stale(LIB, objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp"] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr}")
        os.replace(LIB + ".tmp", LIB)
    probe_src = os.path.join(PROBE_DIR, "probe.hip")
    if force or _stale(PROBE_LIB, [probe_src, os.path.join(PROBE_DIR, "ems_probe.h")] + hdrs):
        cmd = [HIPCC] + FLAGS + ["-shared", probe_src, "-o", PROBE_LIB + ".tmp"]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on probe.hip:\n{r.stderr}")
        os.replace(PROBE_LIB + ".tmp", PROBE_LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
