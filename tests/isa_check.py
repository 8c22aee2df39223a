"""Static check on the ISA that hipcc generates for the library's own kernels.

The pipelined lookup / merge kernels issue their LDS fragment reads through inline asm and
wait for them by hand.  Between such a read and the MFMA that consumes its data, nothing
else may touch the destination registers: a register copy inserted by the compiler there
would move a value that has not arrived yet.  The compiler is free to do that, so the
build is checked rather than trusted."""

import os
import re
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_18736_amd", "csrc")


def device_asm(source: str) -> str:
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-S",
               os.path.join(CSRC, source), "-o", out]
        subprocess.run(cmd, check=True, capture_output=True)
        return open(out).read()


def _regs(text: str):
    regs = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        regs.add(int(m.group(1)))
    return regs


def kernels(asm: str):
    """name -> list of instruction lines and local labels (`.LBBn_m:`), in program order"""
    out, name = {}, None
    for line in asm.split("\n"):
        m = re.match(r"^(_Z\w+):\s*(;.*)?$", line)
        if m:
            name = m.group(1)
            out[name] = []
            continue
        if name is None:
            continue
        if re.match(r"^\.Lfunc_end", line):  # (an early exit puts an s_endpgm in the middle of a kernel)
            name = None
            continue
        m = re.match(r"^(\.LBB\w+):", line)
        if m:
            out[name].append(m.group(1) + ":")
        elif re.match(r"^\s+[a-z]", line):
            out[name].append(line.strip())
    return out


def inflight_violations(lines):
    """For every hand-written `ds_read_b128 v[a:b], vN offset:K` find the first later MFMA (in program
    order) that reads v[a:b]; any other instruction in between that reads or writes those registers is
    a violation.  The same read met again first (the other arm of a branch) ends the search: it is
    checked on its own.  Program order is how the reads, their waits and their MFMAs are laid out;
    branches in between only skip parts of it."""
    bad = []
    for i, line in enumerate(lines):
        m = re.match(r"ds_read_b128 v\[(\d+):(\d+)\], v(\d+) offset:\S+ ; hand-scheduled", line)
        if not m:
            continue
        dst = set(range(int(m.group(1)), int(m.group(2)) + 1))
        for j in range(i + 1, min(len(lines), i + 400)):
            other = lines[j]
            if other.endswith(":") or other == line:
                if other == line:
                    break
                continue
            if other.startswith("v_mfma"):
                ops = other.split(";")[0].split(None, 1)[1].split(", ")
                if _regs(", ".join(ops[1:3])) & dst:
                    break
                if _regs(ops[0]) & dst or _regs(ops[3]) & dst:
                    bad.append((line, other))
                    break
                continue
            if other.startswith(("s_", "global_load_lds")):
                continue
            if other.startswith("ds_read_b128"):
                # other reads may reuse the address register, never the data registers
                if _regs(other.split(",")[0]) & dst:
                    bad.append((line, other))
                    break
                continue
            if _regs(other) & dst:
                bad.append((line, other))
                break
    return bad


def agpr_users_not_hand_placed(lines):
    """In a kernel whose accumulators sit at fixed AGPRs (instructions tagged `hand-placed`), the
    compiler must not use any AGPR itself: it does not know that they hold live values."""
    if not any("hand-placed" in l for l in lines):
        return []
    return [l for l in lines if re.search(r"\ba\[\d+:\d+\]|\ba\d+\b|accvgpr", l.split(";")[0]) and "hand-placed" not in l]


def early_accumulator_reads(lines, distance=12):
    """A hand-placed v_accvgpr_read of aN must come at least `distance` instructions after the last
    MFMA that wrote aN (the compiler inserts no wait states for instructions it cannot see into)."""
    bad = []
    last_write = {}
    for i, line in enumerate(lines):
        if "hand-placed" not in line:
            continue
        m = re.match(r"v_mfma\S* a\[(\d+|0x[0-9a-f]+):(\d+|0x[0-9a-f]+)\]", line)
        if m:
            for r in range(int(m.group(1), 0), int(m.group(2), 0) + 1):
                last_write[r] = i
            continue
        m = re.match(r"v_accvgpr_read_b32 v\d+, a\[(\d+|0x[0-9a-f]+)\]", line)
        if m and i - last_write.get(int(m.group(1), 0), -10 ** 9) < distance:
            bad.append(line)
    return bad


def fixed_fragment_users_not_hand_placed(lines, first=208):
    """The wide kernel keeps its MFMA operand fragments in v[first .. 255] by hand; the compiler's
    own instructions must stay below."""
    if not any(l.startswith("ds_read_b128") and "hand-placed" in l for l in lines):
        return []
    return [l for l in lines if "hand-placed" not in l and not l.endswith(":")
            and any(r >= first for r in _regs(l.split(";")[0]))]


def private_segment_sizes(asm: str):
    """kernel name -> bytes of per-lane scratch memory the compiler gave it (0 = everything in registers)"""
    return {m.group(1): int(m.group(2)) for m in re.finditer(r"\.set (\S+)\.private_seg_size, (\d+)", asm)}
