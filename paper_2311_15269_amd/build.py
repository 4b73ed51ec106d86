"""Builds the HIP library (gfx950) in-tree with hipcc."""
import glob
import os
import re
import shutil
import subprocess
import tempfile

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libtessel_hip.so")
SOURCES = ["tessel_kernels.hip", "tessel_api.cpp"]
HEADERS = ["tessel_device.h", os.path.join("..", "..", "include", "tessel.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
    # packed FP32 instructions are kept out of every device code object of this build
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > built for f in SOURCES + HEADERS)


def misaligned_scalar_loads(asm):
    """Scalar loads of the device code whose address is not visibly a multiple of four: a register offset, or a base
    that was computed from anything but an index shifted left by two or more.  The scalar memory path drops the low
    two bits of the base, so `base + i` with a byte index i, to which the compiler once added `3 i` as the offset of a
    load of word i, reads the wrong word.  (Seen in a variant of the completion kernel that read its per-type
    tables from global memory; the kernels keep such tables in LDS.)  Returns the offending lines."""
    lines = asm.split("\n")
    bad = []
    for n, line in enumerate(lines):
        m = re.search(r"\bs_(?:buffer_)?load_\w+\s+\S+,\s+s\[(\d+):\d+\],\s*(\S+)", line)
        if not m:
            continue
        if re.match(r"s\d+", m.group(2)):                       # register offset
            bad.append("%d: %s" % (n + 1, line.strip()))
            continue
        base = m.group(1)
        for k in range(n - 1, max(0, n - 14), -1):
            t = lines[k]
            if t.startswith(".L") or re.match(r"^\S+:", t):     # start of the basic block: the base came in whole
                break
            if re.search(r"\b(?:s_add_u32|v_readfirstlane_b32)\s+s%s\b" % base, t):
                before = "\n".join(lines[max(0, k - 6):k])
                if not re.search(r"s_lshl_b64\s+s\[\d+:\d+\],\s*s\[\d+:\d+\],\s*[2-9]\b", before):
                    bad.append("%d: %s" % (n + 1, line.strip()))
                break
    return bad


def build_library(force=True, verbose=False, check=True):
    """hipcc --offload-arch=gfx950 ... -> paper_2311_15269_amd/libtessel_hip.so.  With `check` the device assembly
    the compiler leaves behind is scanned for scalar loads at addresses that may not be word aligned."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = tempfile.mkdtemp(prefix="tessel_build_")
    try:
        out = os.path.join(tmp, "libtessel_hip.so")
        cmd = [hipcc] + HIPCC_FLAGS + (["-save-temps=obj"] if check else []) + [os.path.join(CSRC, f) for f in SOURCES] + ["-o", out]
        if verbose:
            print(" ".join(cmd))
        subprocess.check_call(cmd, cwd=tmp)
        if check:
            listings = glob.glob(os.path.join(tmp, "*gfx950*.s"))
            if not listings:
                raise RuntimeError("no device assembly found to check")
            for path in listings:
                bad = misaligned_scalar_loads(open(path).read())
                if bad:
                    raise RuntimeError("scalar loads at possibly unaligned addresses in %s:\n%s" % (os.path.basename(path), "\n".join(bad[:10])))
        shutil.move(out, LIB)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
