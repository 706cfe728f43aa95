"""Builds libdynamix.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

The streaming pass is instantiated for every K in 1..64 and the three storage types, and again
for K in 1..32 with each of the two optimizer updates that carry state; the instantiations are
split over 48 translation units of eight kernels that compile in parallel.
Run as `python -m paper_2510_08522_amd.build`.
"""
import os
import re
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
    for opt in (0, 1, 2):
        for dt in (0, 1, 2):
            for lo in range(1, 65 if opt == 0 else 33, 8):
                jobs.append((os.path.join(CSRC, "stream_pass_inst.hip"),
                             os.path.join(OBJ, "stream_pass_%d_%d_%d.o" % (opt, dt, lo)),
                             ["-DDYNAMIX_INST_OPT=%d" % opt, "-DDYNAMIX_INST_DT=%d" % dt,
                              "-DDYNAMIX_INST_LO=%d" % lo]))
    jobs.append((os.path.join(CSRC, "final_reduce.hip"), os.path.join(OBJ, "final_reduce.o"), []))
    jobs.append((os.path.join(CSRC, "cycle.hip"), os.path.join(OBJ, "cycle.o"), []))
    jobs.append((os.path.join(CSRC, "hbm_probe.hip"), os.path.join(OBJ, "hbm_probe.o"), []))
    jobs.append((os.path.join(CSRC, "wide_pass.hip"), os.path.join(OBJ, "wide_pass.o"), []))
    jobs.append((os.path.join(CSRC, "policy.cpp"), os.path.join(OBJ, "policy.o"), []))
    jobs.append((os.path.join(CSRC, "api.hip"), os.path.join(OBJ, "api.o"), []))
    return jobs


_KERNEL = re.compile(r"stream_pass_kernelILi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)E")


_WIDE_KERNEL = re.compile(r"wide_pass_kernelILi(\d+)E")


def _bank_registers(K, dtype, U, opt=0):
    """Accumulation registers the streaming pass uses on purpose (its two register banks): the
    same arithmetic as Shape<> in csrc/stream_pass.h."""
    if K > 44:
        return 0
    LW, kBlock, stage = (4 if K <= (32 if opt == 0 else 24) else 2), 256, 152 * 1024
    Q = (1 if dtype == 0 else 2)
    slots = stage // (kBlock * LW * 4)
    per_tile_slots = U * Q * (1 + opt)          # a parked tile holds one vector per output stream
    per_tile = per_tile_slots * LW
    first = (slots // per_tile_slots) * per_tile
    second = (256 - first) // per_tile * per_tile
    return first + second


def _check_resources(remarks, src):
    """The streaming pass must not spill vector registers and must not have values moved into
    accumulation registers by the compiler (instantiations built that way have returned wrong
    sums on gfx950); the only accumulation registers allowed are those of its explicit bank.
    Returns the kernels that reserve a private segment without spilling a vector register (the
    compiler sometimes keeps an unused slot per register that carries spilled scalars): their
    code has to be looked at, see _uses_scratch."""
    name, bad, reserved = None, [], []
    scratch = {}
    for line in remarks.splitlines():
        if "Function Name:" in line:
            m = _KERNEL.search(line)
            name = tuple(int(x) for x in m.groups()) if m else None
            w = _WIDE_KERNEL.search(line)
            if w:   # the two-sweep kernel (K > 64, no banks): named (65, dtype, 1, 0) here
                name = (65, int(w.group(1)), 1, 0)
        elif name is not None:
            m = re.search(r"remark:\s+(AGPRs|ScratchSize \[bytes/lane\]|VGPRs Spill): (\d+)", line)
            if not m:
                continue
            what, value = m.group(1), int(m.group(2))
            if what == "AGPRs" and value != _bank_registers(*name):
                bad.append("K=%d dtype=%d opt=%d: %d accumulation registers, expected %d"
                           % (name[0], name[1], name[3], value, _bank_registers(*name)))
            elif what.startswith("Scratch") and value != 0:
                scratch[name] = value
            elif what == "VGPRs Spill" and value != 0:
                bad.append("K=%d dtype=%d opt=%d: %d vector registers spilled" % (name[0], name[1], name[3], value))
    spilled = {b.split(":")[0] for b in bad if "spilled" in b}
    for name, value in scratch.items():
        if "K=%d dtype=%d opt=%d" % (name[0], name[1], name[3]) in spilled:
            bad.append("K=%d dtype=%d opt=%d: %d bytes of scratch" % (name[0], name[1], name[3], value))
        else:
            reserved.append(name)
    if bad:
        raise RuntimeError("register allocation of %s is not as required:\n  %s"
                           % (os.path.basename(src), "\n  ".join(bad)))
    return reserved


def _uses_scratch(assembly):
    """Whether generated code (text, as written by hipcc -S for gfx950, where every access to the
    private segment is a scratch_ instruction) touches the private segment."""
    return re.search(r"^\s+scratch_", assembly, re.MULTILINE) is not None


def _compile(job):
    src, obj, defs = job
    cmd = [HIPCC] + FLAGS + defs + ["-c", src, "-o", obj]
    check = src.endswith("stream_pass_inst.hip") or src.endswith("wide_pass.hip")
    if check:
        cmd.append("-Rpass-analysis=kernel-resource-usage")
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l]
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), "\n".join(lines)))
    if check:
        reserved = _check_resources(r.stdout, src)
        if reserved:
            # a private segment without a spilled vector register: the code must not touch it
            asm = obj[:-2] + ".s"
            a = subprocess.run([HIPCC] + FLAGS + defs + ["-S", "--cuda-device-only", src, "-o", asm],
                               stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            if a.returncode != 0:
                raise RuntimeError("hipcc -S failed for %s" % src)
            with open(asm) as fh:
                text = fh.read()
            os.remove(asm)
            if _uses_scratch(text):
                raise RuntimeError("register allocation of %s is not as required: scratch is "
                                   "accessed (K, dtype, unroll: %s)" % (os.path.basename(src), reserved))
        lines = [l for l in lines if "remark:" not in l and "Rpass-analysis" not in l]
    return "\n".join(lines)


def _check_static_scratch():
    """The static device array of the allocation-free entry point is looked up by name at run
    time (hipGetSymbolAddress), and a lookup that fails aborts the process inside the runtime: the
    array must be a global symbol of the device code (the compiler makes it one because host code
    names it; with a `used` attribute on it, it does not)."""
    src, asm = os.path.join(CSRC, "api.hip"), os.path.join(OBJ, "api_device.s")
    r = subprocess.run([HIPCC] + FLAGS + ["--cuda-device-only", "-S", src, "-o", asm],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed for api.hip:\n" + r.stdout)
    with open(asm) as fh:
        text = fh.read()
    os.remove(asm)
    if not re.search(r"^\s*\.globl\s+_ZL7scratch\s*$", text, re.MULTILINE):
        raise RuntimeError("api.hip: the static scratch array is not a global device symbol")
    if not re.search(r"\.globl\s+_ZL7scratch\s*\n\s*\.p2align\s+8\b", text):
        raise RuntimeError("api.hip: the static scratch array is not 256-byte aligned")


def build(verbose=False, workers=None):
    """Compile every unit and link the shared library; always recompiles."""
    os.makedirs(OBJ, exist_ok=True)
    jobs = _jobs()
    workers = workers or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=workers) as ex:
        checked = ex.submit(_check_static_scratch)
        for out in ex.map(_compile, jobs):
            if verbose and out.strip():
                print(out)
        checked.result()
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + [j[1] for j in jobs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
