"""Build libsage.so (HIP, gfx950 only) in-tree with hipcc.

The quantiser translation unit is compiled with -ffp-contract=off because its
binary32 steps are defined operation by operation; nothing is compiled with
fast-math.  Packed FP32 instructions are disabled for all device code.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsage.so")
OBJDIR = os.path.join(HERE, "_build")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
UNITS = [
    ("sage_quant.hip", ["-ffp-contract=off"]),
    ("sage_attn.hip", []),
    ("sage_api.hip", []),
]


def sources():
    out = [os.path.join(CSRC, u) for u, _ in UNITS]
    out.append(os.path.join(CSRC, "sage_internal.h"))
    out.append(os.path.join(os.path.dirname(HERE), "include", "sage.h"))
    return out


def is_current() -> bool:
    return os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in sources())


def build(verbose: bool = False) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for unit, extra in UNITS:
        obj = os.path.join(OBJDIR, unit.replace(".hip", ".o"))
        cmd = [hipcc, *COMMON, *extra, "-c", os.path.join(CSRC, unit), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
