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
    """name -> list of instruction lines"""
    out, name = {}, None
    for line in asm.split("\n"):
        m = re.match(r"^(_Z\w+):\s*(;.*)?$", line)
        if m:
            name = m.group(1)
            out[name] = []
            continue
        if name is None:
            continue
        if re.match(r"^\s+s_endpgm", line):
            name = None
            continue
        if re.match(r"^\s+[a-z]", line):
            out[name].append(line.strip())
    return out


def inflight_violations(lines):
    """For every hand-written `ds_read_b128 v[a:b], vN offset:K` find the first later MFMA that reads
    v[a:b]; any other instruction in between that reads or writes those registers is a violation.
    Branches are followed in program order only, which is how the reads and their waits are laid out."""
    bad = []
    for i, line in enumerate(lines):
        m = re.match(r"ds_read_b128 v\[(\d+):(\d+)\], v(\d+) offset:\S+ ; hand-scheduled", line)
        if not m:
            continue
        dst = set(range(int(m.group(1)), int(m.group(2)) + 1))
        for j in range(i + 1, min(len(lines), i + 400)):
            other = lines[j]
            if other.startswith("v_mfma"):
                ops = other.split(None, 1)[1].split(", ")
                srcs = _regs(", ".join(ops[1:3]))
                if srcs & dst:
                    break
                if _regs(ops[0]) & dst or _regs(ops[3]) & dst:
                    bad.append((line, other))
                    break
                continue
            if other.startswith(("s_", "ds_read_b128", "global_load_lds")):
                # other reads may reuse the address register, never the data registers
                if other.startswith("ds_read_b128") and _regs(other.split(",")[0]) & dst:
                    bad.append((line, other))
                    break
                continue
            if _regs(other) & dst:
                bad.append((line, other))
                break
    return bad
