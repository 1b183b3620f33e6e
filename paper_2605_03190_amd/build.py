"""Build step of the HIP extension: hipcc -> libvdcores.so next to this file (gfx950 only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SO = os.path.join(HERE, "libvdcores.so")
SOURCES = [os.path.join(HERE, "csrc", "vdc_kernel.hip"), os.path.join(HERE, "csrc", "vdc_host.cpp"), os.path.join(HERE, "csrc", "vdc_lower.cpp")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
         # packed fp32 arithmetic is kept out of the device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


SO_OBSERVER = os.path.join(HERE, "libvdcores_obs.so")   # profiling build with the observer wave; not used by the product path


def build(verbose=False, observer=False):
    """observer=True builds the instrumented library that stage_latency.py loads (an extra read-only wave per core 0)."""
    cmd = ["/opt/rocm/bin/hipcc"] + FLAGS + (["-DVDC_PROFILE"] if observer else []) + SOURCES + ["-o", SO_OBSERVER if observer else SO]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines()
                    if "packed-fp32-ops" not in l)      # the host pass does not know the device feature
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return SO_OBSERVER if observer else SO


if __name__ == "__main__":
    print(build(verbose=True, observer="--observer" in sys.argv))
