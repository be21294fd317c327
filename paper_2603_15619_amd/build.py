"""Compile the HIP sources under csrc/ for gfx950 into libmoda.so next to this file."""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoda.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    # compiler-generated packed fp32 math is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile(src):
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
    subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], check=True,
                   stderr=subprocess.PIPE if os.environ.get("MODA_QUIET_BUILD") else None)
    return obj


# Sources whose inline assembly owns ALL accumulation registers by name (see
# csrc/moda_fwd_regs.h).  The compiler is not told that they hold live values, so the
# build verifies on the generated assembly that it never touches one itself, and that
# nothing was spilled to scratch memory.
NAMED_ACC_SOURCES = ("moda_fwd_bf16.hip",)
FIRST_NAMED_ACC = 0


def check_named_acc_registers(src) -> None:
    import re

    asm = os.path.join(OBJ, os.path.basename(src)[:-4] + ".s")
    subprocess.run([HIPCC, *FLAGS, "--cuda-device-only", "-S", src, "-o", asm], check=True,
                   stderr=subprocess.DEVNULL)
    in_asm = False
    pat = re.compile(r"\ba(?:\[(\d+):(\d+)\]|(\d+))\b")
    for n, line in enumerate(open(asm), 1):
        if "#ASMSTART" in line:
            in_asm = True
            continue
        if "#ASMEND" in line:
            in_asm = False
            continue
        code = line.split(";")[0]
        if in_asm or not code.strip() or code.lstrip().startswith("."):
            continue
        for m in pat.finditer(code):
            hi = int(m.group(2) or m.group(3))
            if hi >= FIRST_NAMED_ACC:
                raise RuntimeError("%s:%d: compiler-allocated use of a%d collides with the named "
                                   "accumulation registers: %s" % (asm, n, hi, line.strip()))
        if code.strip().startswith(("scratch_", "buffer_store", "buffer_load")) and "off" in code and "s[0:3]" in code:
            raise RuntimeError("%s:%d: register spill to scratch memory: %s" % (asm, n, line.strip()))


def build_libmoda() -> str:
    """Always recompiles every source, then links.  Returns the library path."""
    os.makedirs(OBJ, exist_ok=True)
    for src in sources():
        if os.path.basename(src) in NAMED_ACC_SOURCES:
            check_named_acc_registers(src)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, sources()))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_libmoda())
