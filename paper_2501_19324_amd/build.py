"""Compile the HIP sources of this package into ``librsd.so`` and, with the table checks of every pass
switched on (``-DRSD_DEBUG``), ``librsd_debug.so`` (gfx950 only)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "librsd.so")
LIB_DEBUG = os.path.join(HERE, "librsd_debug.so")
SOURCES = [os.path.join(HERE, "csrc", "rsd.hip")]


def _command(out: str, extra: list) -> list:
    return ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + extra + [
            "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"), "-o", out] + SOURCES


def build(verbose: bool = False) -> str:
    jobs = [(LIB, subprocess.Popen(_command(LIB, []), stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)),
            (LIB_DEBUG, subprocess.Popen(_command(LIB_DEBUG, ["-DRSD_DEBUG"]), stdout=subprocess.PIPE,
                                         stderr=subprocess.STDOUT, text=True))]
    for out, proc in jobs:
        text, _ = proc.communicate()
        msgs = "\n".join(l for l in text.splitlines()
                         if "packed-fp32-ops" not in l)      # the host pass does not know the device feature
        if proc.returncode != 0:
            raise RuntimeError(f"hipcc failed for {os.path.basename(out)}:\n" + msgs)
        if verbose and msgs.strip():
            print(msgs)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
