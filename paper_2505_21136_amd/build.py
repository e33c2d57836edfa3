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
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Rpass-analysis=kernel-resource-usage"]
RESOURCES = os.path.join(OBJDIR, "kernel_resources.txt")
UNITS = [
    ("sage_quant.hip", ["-ffp-contract=off"]),
    ("sage_attn.hip", []),
    ("sage_decode.hip", []),
    ("sage_api.hip", []),
    ("sage_diag.hip", []),
]


def sources():
    out = [os.path.join(CSRC, u) for u, _ in UNITS]
    out.append(os.path.join(CSRC, "sage_internal.h"))
    out.append(os.path.join(CSRC, "sage_attn_device.h"))
    out.append(os.path.join(os.path.dirname(HERE), "include", "sage.h"))
    return out


def is_current() -> bool:
    return os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in sources())


_REMARK = "[-Rpass-analysis=kernel-resource-usage]"


def _is_remark_noise(line: str) -> bool:
    t = line.strip()
    return _REMARK in line or t.startswith("|") or (t[:1].isdigit() and " | " in t) or t.endswith("remarks generated.")


def _resource_usage(compiler_output: str) -> dict:
    """{kernel name: {field: int}} from the resource-usage remarks of one hipcc run."""
    usage, cur = {}, None
    for line in compiler_output.splitlines():
        if _REMARK not in line or "remark:" not in line:
            continue
        body = line.split("remark:", 1)[1].replace(_REMARK, "").strip()
        if body.startswith("Function Name:"):
            cur = usage.setdefault(body.split(":", 1)[1].strip(), {})
        elif cur is not None and ":" in body:
            key, val = body.rsplit(":", 1)
            key = key.split("[")[0].strip()
            try:
                cur[key] = int(val)
            except ValueError:
                pass
    return usage


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
    usage = {}
    for cmd, p in procs:
        out, _ = p.communicate()
        usage.update(_resource_usage(out))
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and not _is_remark_noise(l))
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    with open(RESOURCES, "w") as f:
        for name, u in sorted(usage.items()):
            f.write(f"{name} {u}\n")
    # a kernel that spills registers to scratch memory still computes the right result, only slowly:
    # nothing else would notice, so the build refuses it
    bad = {n: u for n, u in usage.items() if u.get("ScratchSize", 0) or u.get("VGPRs Spill", 0)}
    if bad:
        raise RuntimeError("kernels spill registers to scratch memory: " + repr(bad))
    # (the 4+8 variant at d = 128 is built for fewer wavefronts per SIMD on purpose; in the mangled name its
    # template arguments <128, ..., Q4 = true, SPLIT = false> read "attn_kernelILi128E ... Lb1ELb0EEEv")
    def four_bit_d128(name: str) -> bool:
        return "attn_kernelILi128E" in name and "ELb1ELb0EEEv" in name
    slow = {n: u for n, u in usage.items()
            if "attn_kernel" in n and u.get("Occupancy", 0) < 4 and not four_bit_d128(n)}
    if slow:
        raise RuntimeError("attention kernels below 4 wavefronts per SIMD: " + repr(slow))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
