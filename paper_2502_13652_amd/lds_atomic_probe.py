"""Builds and runs csrc/lds_atomic_probe.hip: the cost of the logits pass's one LDS atomic per logit,
by address pattern (cycles per wavefront instruction and CU).  Needs a GPU.

    python -m paper_2502_13652_amd.lds_atomic_probe
"""
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))


def build():
    exe = os.path.join(_HERE, "lib", "lds_atomic_probe")
    os.makedirs(os.path.dirname(exe), exist_ok=True)
    r = subprocess.run(["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", "-o", exe, os.path.join(_HERE, "csrc", "lds_atomic_probe.hip")],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode:
        print(r.stdout)
        raise RuntimeError("hipcc failed")
    return exe


if __name__ == "__main__":
    sys.exit(subprocess.call([build()]))
