"""Builds libpipedit_attn.so in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpipedit_attn.so")
SOURCES = ["attn_fwd.hip", "attn_fwd_sp.hip", "merge.hip", "layout.hip", "probe.hip", "api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-Wno-inline-asm"]      # the DMA helpers declare m0, a register the compiler reserves, as clobbered


def build_library(verbose: bool = False, host_sanitizers: bool = False) -> str:
    """Compile the library next to this file.  host_sanitizers: build the HOST side (argument
    validation, planner, scheduler) with AddressSanitizer and UndefinedBehaviorSanitizer for a CPU
    test run (load it with the ASan runtime preloaded); device code is built as usual."""
    flags = list(FLAGS)
    if host_sanitizers:
        flags = [f for f in flags if f != "-O3"] + ["-O1", "-g", "-Xarch_host", "-fsanitize=address",
                                                      "-Xarch_host", "-fsanitize=undefined",
                                                      "-Xarch_host", "-fno-omit-frame-pointer"]
    cmd = [HIPCC, *flags, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
