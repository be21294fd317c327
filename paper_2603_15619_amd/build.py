"""Compile the HIP sources under csrc/ for gfx950 into libmoda.so next to this file."""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoda.so")
# the seeded input generator is a library of its own (it holds none of the operator's arithmetic)
SYNTH_SRC = os.path.join(HERE, "synth_csrc", "moda_synth.hip")
SYNTH_LIB = os.path.join(HERE, "libmoda_synth.so")

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
# csrc/moda_fwd_regs.h) between the points where the kernel emits the marker comments
# ACC_ACQUIRE_MARKER and ACC_RELEASE_MARKER.  The compiler is not told that they hold live
# values, so the build verifies on the generated assembly, per kernel and on its
# control-flow graph, that
#   - no instruction that can execute between the two markers touches an accumulation
#     register unless it sits inside one of the hand-written assembly statements,
#   - no hand-written statement that names an accumulation register can execute before
#     the acquire marker or after the release marker (there the registers are the compiler's),
#   - nothing was spilled to scratch memory.
NAMED_ACC_SOURCES = ("moda_fwd_bf16.hip",)
ACC_ACQUIRE_MARKER = "MODA_ACC_REGISTERS_ACQUIRED"
ACC_RELEASE_MARKER = "MODA_ACC_REGISTERS_RELEASED"


def _kernel_bodies(asm_path):
    """Yields (name, [(line_no, text)]) for every function of the assembly file."""
    import re

    name, body = None, []
    for n, line in enumerate(open(asm_path), 1):
        if name is None:
            m = re.match(r"^(_Z\w+):", line)
            if m:
                name, body = m.group(1), []
        elif line.startswith(".Lfunc_end"):
            yield name, body
            name = None
        else:
            body.append((n, line.rstrip("\n")))


def _check_kernel(asm_path, name, body) -> None:
    import re

    acc = re.compile(r"\ba(?:\[\d+:\d+\]|\d+)\b")
    # instruction stream: (line_no, text, hand_written)
    ins, labels, in_asm = [], {}, False
    for n, line in body:
        if "#ASMSTART" in line:
            in_asm = True
            continue
        if "#ASMEND" in line:
            in_asm = False
            continue
        if in_asm and (ACC_RELEASE_MARKER in line or ACC_ACQUIRE_MARKER in line):
            ins.append((n, ACC_RELEASE_MARKER if ACC_RELEASE_MARKER in line else ACC_ACQUIRE_MARKER, True))
            continue
        code = line.split(";")[0].strip()
        if not code:
            continue
        m = re.match(r"^(\.LBB\d+_\d+):", code)
        if m:
            labels[m.group(1)] = len(ins)
            continue
        if code.startswith("."):
            continue
        ins.append((n, code, in_asm))
    def the_marker(text):
        found = [i for i, x in enumerate(ins) if x[1] == text]
        if len(found) != 1:
            raise RuntimeError("%s: %s: expected exactly one %s, found %d" % (asm_path, name, text, len(found)))
        return found[0]

    acquire, marker = the_marker(ACC_ACQUIRE_MARKER), the_marker(ACC_RELEASE_MARKER)

    def successors(i):
        op = ins[i][1].split()[0]
        if op in ("s_setpc_b64", "s_swappc_b64", "s_call_b64") or op.startswith("s_cbranch_i_fork"):
            raise RuntimeError("%s:%d: indirect control flow: %s" % (asm_path, ins[i][0], ins[i][1]))
        if op == "s_endpgm":
            return []
        if op == "s_branch":
            return [labels[ins[i][1].split()[1]]]
        out = [i + 1] if i + 1 < len(ins) else []
        if op.startswith("s_cbranch"):
            out.append(labels[ins[i][1].split()[1]])
        return out

    def reach(start, stop=None):
        seen, todo = set(), [start]
        while todo:
            i = todo.pop()
            if i in seen or i == stop:
                continue
            seen.add(i)
            todo.extend(successors(i))
        return seen

    if marker in reach(0, stop=acquire):
        raise RuntimeError("%s: %s: the release marker can be reached without passing the acquire marker"
                           % (asm_path, name))
    owned = reach(acquire, stop=marker)     # can execute between the markers
    free = reach(0, stop=acquire) | reach(marker)  # before the acquire marker or after the release marker
    for i in sorted(owned):
        n, code, hand = ins[i]
        if not hand and acc.search(code):
            raise RuntimeError("%s:%d: %s: compiler-allocated accumulation register while the named "
                               "ones are live: %s" % (asm_path, n, name, code))
    for i in sorted(free):
        n, code, hand = ins[i]
        if hand and acc.search(code):
            raise RuntimeError("%s:%d: %s: named accumulation register used outside the owned region: %s"
                               % (asm_path, n, name, code))


def check_named_acc_registers(src) -> None:
    asm = os.path.join(OBJ, os.path.basename(src)[:-4] + ".s")
    subprocess.run([HIPCC, *FLAGS, "--cuda-device-only", "-S", src, "-o", asm], check=True,
                   stderr=subprocess.DEVNULL)
    n_kernels = 0
    for name, body in _kernel_bodies(asm):
        _check_kernel(asm, name, body)
        n_kernels += 1
    if n_kernels == 0:
        raise RuntimeError("%s: no kernel found" % asm)
    for line in open(asm):
        if line.startswith("; ScratchSize:") and int(line.split(":")[1]) != 0:
            raise RuntimeError("%s: register spill to scratch memory (%s)" % (asm, line.strip()))


# Kernels whose key loop keeps global -> LDS copies in flight while it computes must not
# touch scratch memory inside that loop: memory operations complete in order, so waiting for a
# reload also waits for the copies (measured on the dK/dV kernel: 1.9 ms with 100 bytes of
# scratch per lane reloaded in the loop, 1.55 ms without).  A value parked in scratch before
# the loops and fetched after them is harmless.
# (source file, substring of the mangled kernel name)
NO_SCRATCH_IN_LOOPS = (("moda_bwd_bf16.hip", "moda_bwd_dkdv_kernel"), ("moda_bwd_bf16.hip", "moda_bwd_dq_kernel"))


def check_no_scratch_in_loops(src, name_part) -> None:
    asm = os.path.join(OBJ, os.path.basename(src)[:-4] + ".s")
    subprocess.run([HIPCC, *FLAGS, "--cuda-device-only", "-S", src, "-o", asm], check=True,
                   stderr=subprocess.DEVNULL)
    scan_scratch_in_key_loops(asm, name_part)


def scan_scratch_in_key_loops(asm, name_part) -> None:
    """Raises if a kernel of assembly file `asm` whose name contains `name_part` touches scratch
    memory inside a loop that issues matrix instructions."""
    import re

    found = 0
    for name, body in _kernel_bodies(asm):
        if name_part not in name:
            continue
        found += 1
        # the compiler annotates every basic block of a loop with the header of its innermost loop;
        # the loops that matter are those that issue matrix instructions (the key loops)
        header, per_line = None, []
        for n, line in body:
            if re.match(r"^(\.LBB\d+_\d+:|; %bb\.\d+:)", line):
                m = re.search(r"Header=(BB\d+_\d+)", line)
                if m:
                    header = m.group(1)
                elif "Loop Header" in line:
                    header = re.match(r"^\.L(BB\d+_\d+):", line).group(1)
                else:
                    header = None
            per_line.append((n, line, header))
        hot = {h for _, line, h in per_line if h and re.match(r"^\s*v_mfma", line)}
        for n, line, h in per_line:
            if h in hot and re.match(r"^\s*scratch_", line):
                raise RuntimeError("%s:%d: %s touches scratch memory inside a key loop: %s"
                                   % (asm, n, name, line.strip()))
    if found == 0:
        raise RuntimeError("%s: no kernel named *%s*" % (asm, name_part))


def build_libmoda() -> str:
    """Always recompiles every source, then links.  Returns the library path."""
    os.makedirs(OBJ, exist_ok=True)
    for src in sources():
        if os.path.basename(src) in NAMED_ACC_SOURCES:
            check_named_acc_registers(src)
        for fname, part in NO_SCRATCH_IN_LOOPS:
            if os.path.basename(src) == fname:
                check_no_scratch_in_loops(src, part)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, sources()))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], check=True)
    os.replace(tmp, LIB)
    build_synth()
    return LIB


def build_synth() -> str:
    """Compiles the device-side input generator into libmoda_synth.so."""
    tmp = SYNTH_LIB + ".tmp.%d" % os.getpid()
    subprocess.run([HIPCC, *FLAGS, "-shared", SYNTH_SRC, "-o", tmp], check=True,
                   stderr=subprocess.PIPE if os.environ.get("MODA_QUIET_BUILD") else None)
    os.replace(tmp, SYNTH_LIB)
    return SYNTH_LIB


if __name__ == "__main__":
    print(build_libmoda())
