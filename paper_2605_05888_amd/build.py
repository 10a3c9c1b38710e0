"""Builds the HIP library (gfx950) in-tree with hipcc.

    python -m paper_2605_05888_amd.build

One translation unit per step; objects are compiled in parallel and linked into
``paper_2605_05888_amd/libmoe_hub.so``.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoe_hub.so")
SOURCES = ["api.hip", "route.hip", "layout.hip", "rowmove.hip", "ffn.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-ffp-contract=off",
    # packed fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


# The grouped GEMM's tall tiles (csrc/grouped_gemm.h, `xa`) keep an operand in vector registers that
# hand-written buffer loads fill while hand-written matrix instructions are still to read them; the
# compiler is not told, and the kernel is correct only as long as it never copies or reuses those
# registers inside the K loop.  That was checked in the generated code of the compilers listed here
# (and is checked on the GPU by the test that reverses every expert segment and expects the same bits).
# Another compiler may schedule differently: read the listing again before adding it.
TESTED_COMPILERS = ("7.2.26015",)


def check_compiler() -> str:
    out = subprocess.run([HIPCC, "--version"], capture_output=True, text=True).stdout
    version = next((l.split(":", 1)[1].strip() for l in out.splitlines() if l.startswith("HIP version")), "unknown")
    if not any(version.startswith(v) for v in TESTED_COMPILERS):
        if os.environ.get("MOE_HUB_UNTESTED_COMPILER") != "1":
            raise RuntimeError(
                f"hipcc reports HIP version {version}; this library was checked with {TESTED_COMPILERS}. "
                "The tall-tile code of csrc/grouped_gemm.h relies on the compiler leaving the registers of "
                "`xa` alone inside the K loop: inspect the listing of grouped_gemm_bf16 (no instruction but "
                "the hand-written buffer loads and v_mfma may touch them), run "
                "tests/test_gpu_parity.py::test_ffn_remainder_rows_riding_with_the_last_full_tile, then add "
                "the version to TESTED_COMPILERS or set MOE_HUB_UNTESTED_COMPILER=1.")
        sys.stderr.write(f"warning: untested hipcc (HIP version {version})\n")
    return version


def _compile(src: str, defines=(), obj_dir: str = OBJ) -> str:
    obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *[f"-D{d}" for d in defines], "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    noise = "is not a recognized feature for this target"
    warn = "\n".join(l for l in r.stderr.splitlines() if l.strip() and noise not in l)
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(verbose: bool = True, defines=(), out: str = LIB) -> str:
    """Builds the library.  `defines` (NAME=VALUE strings) and `out` give a variant build next to the
    default one, for timing two builds against each other (load it with MOE_HUB_LIBRARY=<out>)."""
    check_compiler()
    obj_dir = OBJ if out == LIB else OBJ + "_" + os.path.splitext(os.path.basename(out))[0]
    os.makedirs(obj_dir, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda src: _compile(src, defines, obj_dir), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    subprocess.run(cmd, check=True)
    if verbose:
        print(f"built {out}")
    return out


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "moe_hub.h"))
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("-D", dest="defines", action="append", default=[], help="NAME=VALUE for the preprocessor")
    ap.add_argument("--out", default=LIB)
    a = ap.parse_args()
    build(defines=a.defines, out=os.path.abspath(a.out))
