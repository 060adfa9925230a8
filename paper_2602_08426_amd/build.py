"""Builds libprism.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libprism.so")
SOURCES = ["prism_estimate.hip", "prism_attn.hip"]
# bench-only probes of the machine's achievable peaks (bench.py --peaks); not part of libprism
PEAKS_LIB_PATH = os.path.join(HERE, "libprism_peaks.so")
PEAKS_SOURCES = ["prism_peaks.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # no packed-fp32 VALU code generation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # queue pulls stay plain returning atomics whose result is waited for where it is used
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
]


def _compile(sources: list[str], out_path: str, verbose: bool, extra_flags: list[str] | None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *(extra_flags or []), "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in sources], "-o", out_path]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out_path


def build_library(verbose: bool = False, extra_flags: list[str] | None = None) -> str:
    """Compile every HIP source into paper_2602_08426_amd/libprism.so (and the bench-only
    libprism_peaks.so beside it) and return the path of libprism.so."""
    # the hand-scheduled row loop of the 64-queries-per-wave attention kernel is generated
    gen = subprocess.run([sys.executable, os.path.join(CSRC, "gen_attn_w64.py"),
                          os.path.join(CSRC, "prism_attn_w64_body.inc")], capture_output=True, text=True)
    if gen.returncode != 0:
        raise RuntimeError(f"gen_attn_w64.py failed:\n{gen.stderr}")
    if verbose:
        print(gen.stderr.strip(), flush=True)
    _compile(PEAKS_SOURCES, PEAKS_LIB_PATH, verbose, None)
    return _compile(SOURCES, LIB_PATH, verbose, extra_flags)


SELECT_ABLATION_BITS = {"select_noscores": 1, "select_nosearch": 2, "select_norefetch": 4}


def build_ablation(experiment: str, out_path: str, verbose: bool = False) -> str:
    """A measurement-only variant of libprism.so that leaves parts out; results are wrong by construction,
    control flow and bounds are unchanged.  `experiment` is a space-separated list of
      nosoft nocopy nowait nobar_mid nobar_end   parts of the 64-queries-per-wave attention row loop
                                                 (PRISM_W64_EXPERIMENT of gen_attn_w64.py),
      select_noscores select_nosearch select_norefetch   parts of the selection kernel
                                                 (PRISM_SELECT_ABLATION of prism_estimate.hip).
    The generated loop and the library go to the given path; the product library is not touched."""
    import shutil
    import tempfile
    with tempfile.TemporaryDirectory() as tmp:
        for name in os.listdir(CSRC):
            if name.endswith((".hip", ".h")):
                shutil.copy(os.path.join(CSRC, name), tmp)
        env = dict(os.environ, PRISM_W64_EXPERIMENT=experiment)
        gen = subprocess.run([sys.executable, os.path.join(CSRC, "gen_attn_w64.py"),
                              os.path.join(tmp, "prism_attn_w64_body.inc")], capture_output=True, text=True, env=env)
        if gen.returncode != 0:
            raise RuntimeError(f"gen_attn_w64.py failed:\n{gen.stderr}")
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        bits = sum(SELECT_ABLATION_BITS.get(tok, 0) for tok in experiment.split())
        cmd = [hipcc, *HIPCC_FLAGS, f"-DPRISM_SELECT_ABLATION={bits}", "-I", os.path.join(ROOT, "include"), "-I", tmp,
               *[os.path.join(tmp, s) for s in SOURCES], "-o", out_path]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed ({res.returncode}):\n{res.stderr}")
    return out_path


if __name__ == "__main__":
    if len(sys.argv) == 4 and sys.argv[1] == "--ablation":
        print(build_ablation(sys.argv[2], sys.argv[3], verbose=True))
    else:
        print(build_library(verbose=True))
