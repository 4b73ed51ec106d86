"""Builds the HIP library (gfx950) in-tree with hipcc."""
import concurrent.futures
import glob
import os
import re
import shutil
import subprocess
import tempfile

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libtessel_hip.so")
SOURCES = ["tessel_kernels.hip", "tessel_wide.hip", "tessel_api.cpp"]
HEADERS = ["tessel_device.h", os.path.join("..", "..", "include", "tessel.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    # packed FP32 instructions are kept out of every device code object of this build
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > built for f in SOURCES + HEADERS)


def _const(tok):
    try:
        return int(tok, 0)
    except ValueError:
        return None


def _word_aligned(reg, block, upto, depth=0, unknown=True):
    """Is scalar register `reg` (a number) visibly a multiple of four at line `upto` of the basic block `block`?
    Follows its latest definition inside the block: shifts left by two or more, multiples of four, sums of such;
    a register the block does not define came in whole (`unknown`: a pointer argument or a value checked elsewhere;
    not assumed of the factors of a product)."""
    if depth > 8:
        return False
    for k in range(upto - 1, -1, -1):
        t = block[k]
        m = re.search(r"\bs_lshl_b64\s+s\[(\d+):(\d+)\],\s*\S+,\s*(\S+)", t)
        if m and int(m.group(1)) <= reg <= int(m.group(2)):
            c = _const(m.group(3))
            return reg > int(m.group(1)) or (c is not None and c >= 2)
        m = re.search(r"\b(s_\w+|v_readfirstlane_b32|v_readlane_b32)\s+s(\d+),\s*(.*)$", t)
        if not m or int(m.group(2)) != reg:
            m2 = re.search(r"\bs_(?:buffer_)?load_\w+\s+s\[(\d+):(\d+)\]", t)
            if m2 and int(m2.group(1)) <= reg <= int(m2.group(2)):
                return True                                      # a pointer read from memory whole
            continue
        op, args = m.group(1), [a.strip() for a in m.group(3).split(",")]

        def ok(a, unknown=True):
            c = _const(a)
            if c is not None:
                return c % 4 == 0
            r = re.match(r"s(\d+)$", a)
            return bool(r) and _word_aligned(int(r.group(1)), block, k, depth + 1, unknown)
        if op == "v_readlane_b32":                               # a spilled scalar register coming back
            return True
        if op in ("s_lshl_b32",):
            c = _const(args[1]) if len(args) > 1 else None
            return c is not None and c >= 2
        if op in ("s_mul_i32",):
            return len(args) == 2 and (ok(args[0], False) or ok(args[1], False))
        if op in ("s_add_u32", "s_add_i32", "s_sub_u32", "s_sub_i32"):
            return len(args) == 2 and ok(args[0]) and ok(args[1])
        if op in ("s_mov_b32",):
            return len(args) == 1 and ok(args[0])
        return False
    return unknown


def misaligned_scalar_loads(asm):
    """Scalar loads of the device code whose address is not visibly a multiple of four: a register offset, or a base
    computed in its basic block from anything but indices shifted left by two or more or multiplied by a multiple of
    four.  The scalar memory path drops the low two bits of the base, so `base + i` with a byte index i, to which the
    compiler once added `3 i` as the offset of a load of word i, reads the wrong word.  (Seen in a variant of the
    completion kernel that read its per-type tables from global memory; the kernels keep such tables in LDS.)
    Returns the offending lines."""
    lines = asm.split("\n")
    bad = []
    start = 0                                                    # first line of the current basic block
    for n, line in enumerate(lines):
        if line.startswith(".L") or re.match(r"^\S+:", line):
            start = n + 1
            continue
        m = re.search(r"\bs_(?:buffer_)?load_\w+\s+\S+,\s+s\[(\d+):\d+\],\s*(\S+)", line)
        if not m:
            continue
        if re.match(r"s\d+", m.group(2)):                       # register offset
            bad.append("%d: %s" % (n + 1, line.strip()))
            continue
        if not _word_aligned(int(m.group(1)), lines[start:n], n - start):
            bad.append("%d: %s" % (n + 1, line.strip()))
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
        # one object per source, compiled side by side (each in a folder of its own, which also takes what
        # -save-temps leaves behind), then one link
        def compile_one(src):
            work = os.path.join(tmp, os.path.splitext(src)[0])
            os.makedirs(work)
            obj = os.path.join(work, os.path.splitext(src)[0] + ".o")
            cmd = [hipcc] + HIPCC_FLAGS + (["-save-temps=obj"] if check else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd))
            subprocess.check_call(cmd, cwd=work)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        link = [hipcc, "--offload-arch=gfx950", "--hip-link", "-shared", "-fPIC"] + objs + ["-o", out]
        if verbose:
            print(" ".join(link))
        subprocess.check_call(link, cwd=tmp)
        if check:
            listings = glob.glob(os.path.join(tmp, "*", "*gfx950*.s"))
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
