"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libnimble_hip.so")
SOURCES = ["nimble_host.cpp", "nimble_vm.cpp", "nimble_kernels.hip"]  # the .h files under csrc/ hold the kernels


def hipcc_command(out: str = LIB):
    return [
        "hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
        # keep the compiler from forming packed-fp32 instructions
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        *[os.path.join(CSRC, s) for s in SOURCES],
        "-o", out,
    ]


def build_library(verbose: bool = False) -> str:
    proc = subprocess.run(hipcc_command(), stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for l in proc.stdout.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    return LIB


def device_assembly() -> str:
    """The gfx950 assembly of the kernels, as text (same flags as the library)."""
    import tempfile
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "kernels.s")
        cmd = [
            "hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "--cuda-device-only", "-S",
            "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            os.path.join(CSRC, "nimble_kernels.hip"), "-o", out,
        ]
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc -S failed:\n" + proc.stdout[-4000:])
        with open(out) as f:
            return f.read()


def _agprs(text: str) -> set:
    import re
    regs = set()
    for lo, hi in re.findall(r"\ba\[(\d+):(\d+)\]", text):
        regs.update(range(int(lo), int(hi) + 1))
    regs.update(int(r) for r in re.findall(r"\ba(\d+)\b", text))
    return regs


def asm_mfma_findings(asm: str, wait_states: int = 18):
    """Checks of the compiler's output around the MFMAs that the kernels write as volatile
    statements.  The compiler does not know that those are matrix instructions and adds no wait
    states behind them, so anything else that touches their result registers too soon reads (or
    overwrites) them before the matrix core has written them.  Returns (hazards, spills):
      hazards: (kernel, line number, instruction) of every instruction outside such statements
               that names an accumulation register written by such an MFMA fewer than
               `wait_states` issue slots earlier (an MFMA counts 8 slots, s_nop N counts N+1);
      spills:  (kernel, block label, count) of scratch accesses in basic blocks that hold such MFMAs
               and sit at the deepest loop level at which the kernel has any (register spills inside
               a main loop; a spill in a stage the compiler peeled off in front of the loop, once per
               tile, is not one).  Blocks are told apart by their labels and by the compiler's
               "%bb.N" comments for blocks reached by falling through; the loop level is the one the
               compiler prints behind either."""
    import re
    hazards, spills = [], []
    kernel, block, in_stmt = None, None, False
    block_mfma, block_scratch, block_depth = 0, 0, 0
    recent = []  # [age in issue slots, registers written] per statement-MFMA still within reach
    blocks = []  # of the current kernel: (label, loop level, MFMAs, scratch accesses)

    def close_block():
        if block_mfma:
            blocks.append((block, block_depth, block_mfma, block_scratch))

    def close_kernel():
        close_block()
        if blocks:
            deepest = max(b[1] for b in blocks)
            spills.extend((kernel, b[0], b[3]) for b in blocks if b[1] == deepest and b[3])
        blocks.clear()

    for no, line in enumerate(asm.split("\n"), 1):
        t = line.strip()
        m = re.match(r"^(_Z\w+):", line)
        if m:
            close_kernel()
            kernel, block, block_mfma, block_scratch, block_depth, recent = m.group(1), "entry", 0, 0, 0, []
            continue
        m = re.match(r"^(\.LBB\w+):", line) or re.match(r"^; (%bb\.\d+):", line)
        if m:
            close_block()
            block, block_mfma, block_scratch = m.group(1), 0, 0
            d = re.search(r"Depth=(\d+)", line)
            block_depth = int(d.group(1)) if d else 0
            continue
        if t.startswith(";") and "Loop Header: Depth=" in t and not block_mfma and not block_scratch:
            block_depth = int(re.search(r"Depth=(\d+)", t).group(1))  # second comment line of a loop header
            continue
        if t.startswith(";;#ASMSTART"):
            in_stmt = True
            continue
        if t.startswith(";;#ASMEND"):
            in_stmt = False
            continue
        if not t or t[0] in ";." or t.endswith(":"):
            continue
        if t.startswith("v_mfma"):
            recent = [[age + 8, regs] for age, regs in recent]
            if in_stmt:
                block_mfma += 1
                recent.append([0, _agprs(t.split(None, 1)[1].split(",")[0])])
            continue
        if t.startswith("s_nop"):
            n = int(t.split()[1], 0) + 1
            recent = [[age + n, regs] for age, regs in recent]
            continue
        if t.startswith("scratch_"):
            block_scratch += 1
        touched = _agprs(t)
        if touched:
            for age, regs in recent:
                if age < wait_states and touched & regs:
                    hazards.append((kernel, no, t))
                    break
        recent = [[age + 1, regs] for age, regs in recent if age + 1 < 4 * wait_states]
    close_kernel()
    return hazards, spills


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "nimble.h"), os.path.join(ROOT, "include", "nimble_vm.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build_library(verbose=True))
