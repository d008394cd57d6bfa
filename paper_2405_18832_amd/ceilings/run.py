"""Practical ceilings of the GPU that the roofline fractions are read against: builds the three stand-alone
probes of this folder for gfx950 and runs them (needs a GPU).  `python -m paper_2405_18832_amd.ceilings.run`
prints their output; `build()` alone compiles them (no GPU needed)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
PROBES = ["mfma_power", "l2_copy_patterns", "hbm_few_cus"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build() -> list:
    outs = []
    for p in PROBES:
        exe = os.path.join(HERE, p + ".exe")
        r = subprocess.run([HIPCC, *FLAGS, "-o", exe, os.path.join(HERE, p + ".hip")], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {p}.hip:\n" + "\n".join(
                l for l in r.stderr.splitlines() if "is not a recognized feature" not in l))
        outs.append(exe)
    return outs


def main() -> int:
    for exe in build():
        print(f"== {os.path.basename(exe)}", flush=True)
        r = subprocess.run([exe], timeout=300)
        if r.returncode != 0:
            return r.returncode
    return 0


if __name__ == "__main__":
    sys.exit(main())
