"""Builds libdynamix.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

The streaming pass is instantiated for every K in 1..64 and the three storage types; the
instantiations are split over 24 translation units that compile in parallel.
Run as `python -m paper_2510_08522_amd.build`.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libdynamix.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         # packed fp32 forms must not be generated on this target
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _jobs():
    jobs = []
    for dt in (0, 1, 2):
        for lo in range(1, 65, 8):
            jobs.append((os.path.join(CSRC, "stream_pass_inst.hip"),
                         os.path.join(OBJ, "stream_pass_%d_%d.o" % (dt, lo)),
                         ["-DDYNAMIX_INST_DT=%d" % dt, "-DDYNAMIX_INST_LO=%d" % lo]))
    jobs.append((os.path.join(CSRC, "final_reduce.hip"), os.path.join(OBJ, "final_reduce.o"), []))
    jobs.append((os.path.join(CSRC, "cycle.hip"), os.path.join(OBJ, "cycle.o"), []))
    jobs.append((os.path.join(CSRC, "api.hip"), os.path.join(OBJ, "api.o"), []))
    return jobs


def _compile(job):
    src, obj, defs = job
    cmd = [HIPCC] + FLAGS + defs + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose=False, workers=None):
    """Compile every unit and link the shared library; always recompiles."""
    os.makedirs(OBJ, exist_ok=True)
    jobs = _jobs()
    workers = workers or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=workers) as ex:
        for out in ex.map(_compile, jobs):
            if verbose and out.strip():
                print(out)
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + [j[1] for j in jobs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
