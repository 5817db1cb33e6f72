"""Compile the HIP sources into paper_2511_21702_amd/libcsvdecode.so for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcsvdecode.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["csv_step.hip", "csv_index.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-FP32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
        if verbose and r.stderr.strip():
            keep = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and "is not a recognized feature" not in l]
            if keep:
                print("\n".join(keep), file=sys.stderr)
        return obj

    with ThreadPoolExecutor(len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


def build_oracle() -> None:
    """Compile whatever C the CPU oracle holds (it is plain numpy at present: nothing to compile)."""
    odir = os.path.join(ROOT, "oracle")
    for f in sorted(os.listdir(odir)):
        if f.endswith(".c"):
            out = os.path.join(odir, "lib" + f[:-2] + ".so")
            r = subprocess.run(["gcc", "-O2", "-fPIC", "-shared", os.path.join(odir, f), "-o", out, "-lm"],
                               capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(f"gcc failed for {f}:\n{r.stdout}\n{r.stderr}")


if __name__ == "__main__":
    build()
    build_oracle()
