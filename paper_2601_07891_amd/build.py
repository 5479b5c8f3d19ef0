"""Build libkvzap.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

try:
    from .isa_lint import lint_scorer_asm
except ImportError:        # run as a script
    from isa_lint import lint_scorer_asm

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libkvzap.so")
CEILINGS_PATH = os.path.join(HERE, "kvzap_ceilings")
SOURCES = ["api.hip", "mask.hip", "compact.hip", "score_linear.hip", "score_mlp.hip",
           "decode.hip", "attend.hip", "paged.hip", "topk.hip", "teacher.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC,
         "-Wall", "-Wno-unused-command-line-argument"]


# sources whose device assembly is checked after compilation (see isa_lint.py)
LINTED = {"score_mlp.hip"}


def _quiet(stderr: str) -> str:
    # hipcc's host pass does not know the device-only target feature and says so for every
    # function; anything else is passed on
    return "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l).strip()


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    tmp = None
    if src in LINTED:     # keep the intermediate device assembly of this one compile
        tmp = os.path.join(OBJ_DIR, "lint_" + src.replace(".hip", ""))
        shutil.rmtree(tmp, ignore_errors=True)
        os.makedirs(tmp)
        cmd = [HIPCC, *FLAGS, "-save-temps=obj", "-c", os.path.join(CSRC, src), "-o",
               os.path.join(tmp, os.path.basename(obj))]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    if _quiet(r.stderr):
        sys.stderr.write(_quiet(r.stderr) + "\n")
    if tmp:
        try:
            asm = [f for f in os.listdir(tmp) if f.endswith(".s") and "amdgcn" in f]
            if len(asm) != 1:
                raise RuntimeError(f"expected one device assembly file for {src}, found {asm}")
            with open(os.path.join(tmp, asm[0])) as fh:
                findings = lint_scorer_asm(fh.read())
            bad = {k: v for k, v in findings.items() if v}
            if bad:
                msg = "\n".join(f"{k}: {len(v)} (first: {v[0][1]})" for k, v in bad.items())
                raise RuntimeError(f"{src}: registers of outstanding loads are touched:\n{msg}")
            os.replace(os.path.join(tmp, os.path.basename(obj)), obj)
        finally:
            shutil.rmtree(tmp, ignore_errors=True)
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(6, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB_PATH}")
    return LIB_PATH


def build_ceilings(verbose: bool = True) -> str:
    """On request only (`python -m paper_2601_07891_amd.build --ceilings`): the stand-alone
    calibration program that measures the practical MFMA / HBM ceilings of the GPU it runs on.
    It is not part of the library and the default build leaves it out."""
    cmd = [HIPCC, *FLAGS, os.path.join(CSRC, "ceilings.hip"), "-o", CEILINGS_PATH]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for ceilings.hip:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {CEILINGS_PATH}")
    return CEILINGS_PATH


if __name__ == "__main__":
    if "--ceilings" in sys.argv[1:]:
        build_ceilings()
    else:
        build()
