"""Builds the gfx950 shared libraries in-tree with hipcc (no torch extension machinery)."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_PKG, "csrc")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 VALU forms are switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

LIBRHINO = os.path.join(_PKG, "librhino.so")
LIBSYNTH = os.path.join(_PKG, "workloads", "libsynthfill.so")

RHINO_SOURCES = [os.path.join(_CSRC, f) for f in
                 ("rhino_api.hip", "chain_dp.hip", "chain_gang.hip", "chain_scan.hip", "chain_fused.hip", "backtrack.hip", "reshard.hip", "stage_dp.hip", "stage_fast.hip", "interval_costs.hip", "interval_blocks.hip", "stage_interval.hip", "stage_plans.hip", "cone.hip", "tree.hip", "memory.hip")]
SYNTH_SOURCES = [os.path.join(_PKG, "workloads", "csrc", "synth_fill.hip")]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + r.stdout)
    return r.stdout


def build_all(verbose: bool = False) -> None:
    """Compile both libraries, every time it is called."""
    for out, srcs in ((LIBRHINO, RHINO_SOURCES), (LIBSYNTH, SYNTH_SOURCES)):
        log = _run([HIPCC] + FLAGS + ["-o", out] + srcs)
        if verbose and log.strip():
            print(log)


def build_host_sanitized(out: str) -> str:
    """librhino with its HOST code (argument checks, planners, launch set-up) under the address and
    undefined-behaviour sanitizers; the device code is compiled as usual.  For CPU-side tests only."""
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = [f if f != "-O3" else "-O1" for f in FLAGS] + ["-g"] + san
    _run([HIPCC] + flags + ["-o", out] + RHINO_SOURCES)
    return out


def host_sanitizer_runtime() -> str:
    """The shared AddressSanitizer runtime of the compiler that hipcc drives (to be preloaded by the test process)."""
    return _run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"]).strip().splitlines()[-1]


if __name__ == "__main__":
    build_all(verbose=True)
    print("built", LIBRHINO, LIBSYNTH)
