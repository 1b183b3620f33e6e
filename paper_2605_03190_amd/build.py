"""Build step of the HIP extension: hipcc -> libvdcores.so next to this file (gfx950 only).

The executor kernel exists in several variants (one per family of compute uops) and each takes a minute or more to
compile, so the kernel source is compiled once per variant (-DVDC_PART=i) and once for everything else (-DVDC_SPLIT),
all at the same time, and the objects are linked into one library."""
import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
SO = os.path.join(HERE, "libvdcores.so")
KERNEL = os.path.join(HERE, "csrc", "vdc_kernel.hip")
HOST = [os.path.join(HERE, "csrc", f) for f in ("vdc_host.cpp", "vdc_lower.cpp", "vdc_sched.cpp")]
SOURCES = [KERNEL] + HOST
N_VARIANTS = 9      # kVariants in csrc/vdc_kernel.hip
WAVE_MASK_VARIANTS = (6, 7, 8)     # ... of which these are built with -DVDC_WAVE_MASKS (see Ctl::mask there)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         # packed fp32 arithmetic is kept out of the device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
HIPCC = "/opt/rocm/bin/hipcc"

SO_OBSERVER = os.path.join(HERE, "libvdcores_obs.so")   # profiling build with the observer wave; not used by the product path


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines()
                    if "packed-fp32-ops" not in l)      # the host pass does not know the device feature
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose=False, observer=False):
    """observer=True builds the instrumented library that stage_latency.py loads (an extra read-only wave per core 0;
    one variant of the kernel, one unit)."""
    if observer:
        _run([HIPCC] + FLAGS + ["-shared", "-DVDC_PROFILE"] + SOURCES + ["-o", SO_OBSERVER], verbose)
        return SO_OBSERVER
    tmp = tempfile.mkdtemp(prefix="vdc_build_")
    try:
        jobs = [(["-DVDC_PART=%d" % i] + (["-DVDC_WAVE_MASKS"] if i in WAVE_MASK_VARIANTS else []) + [KERNEL], os.path.join(tmp, "part%d.o" % i))
                for i in range(N_VARIANTS)]
        jobs.append((["-DVDC_SPLIT", KERNEL], os.path.join(tmp, "kernel.o")))
        jobs += [([src], os.path.join(tmp, os.path.basename(src) + ".o")) for src in HOST]
        workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", "0")) or os.cpu_count() or 1))
        with ThreadPoolExecutor(workers) as pool:
            list(pool.map(lambda j: _run([HIPCC] + FLAGS + ["-c"] + j[0] + ["-o", j[1]], verbose), jobs))
        _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + [j[1] for j in jobs] + ["-o", SO], verbose)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return SO


if __name__ == "__main__":
    print(build(verbose=True, observer="--observer" in sys.argv))
