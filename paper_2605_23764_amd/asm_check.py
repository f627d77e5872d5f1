"""Static check of a contract the compiler cannot see (csrc/gemm_bf16.h, register-fed row block of the wide tile).

The block's activation fragments are fetched by plain global loads written as inline assembly, so that they ride the
pipeline's hand-kept `s_waitcnt vmcnt` accounting.  Their destination registers are written by the hardware some time
after the statement, behind the compiler's back: from the request to the wait that retires them (another assembly
statement, `s_waitcnt vmcnt(n)`, which names the registers) no instruction may read or write those registers.  The
source is arranged so that the compiler has no reason to (the window lies inside one loop trip and ends in the naming
wait), but nothing in the language enforces it; this module checks the generated code.

    python -m paper_2605_23764_amd.asm_check        # compiles the device code to assembly and checks it
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))

_RANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_SINGLE = re.compile(r"\bv(\d+)\b")


def _vregs(text: str) -> set:
    regs = set()
    for lo, hi in _RANGE.findall(text):
        regs.update(range(int(lo), int(hi) + 1))
    regs.update(int(r) for r in _SINGLE.findall(_RANGE.sub(" ", text)))
    return regs


def device_assembly() -> str:
    """Device-only assembly of csrc/moe_ffn.hip with the library's own flags."""
    from .build import HIPCC_FLAGS, SOURCES
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "device.s")
        res = subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", *SOURCES, "-o", out], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
        with open(out) as f:
            return f.read()


def check_register_fed_loads(asm: str):
    """Returns (number of assembly loads with register destinations, list of violations).  A violation is
    (line number, instruction, registers) for an instruction between such a load and the next assembly
    `s_waitcnt vmcnt` that touches the load's destination registers."""
    pending = {}          # register -> line of the load that will write it
    n_loads, bad = 0, []
    in_asm = False
    for no, raw in enumerate(asm.splitlines(), 1):
        line = raw.split(";")[0].strip() if not raw.lstrip().startswith(";;#") else raw.strip()
        if line.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if line.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not line or line.startswith(".") or line.endswith(":"):
            if line.startswith(".end_amdhsa_kernel") or line.startswith(".amdhsa_kernel"):
                pending.clear()
            continue
        if in_asm:
            m = re.match(r"global_load_dwordx4\s+v\[(\d+):(\d+)\]\s*,\s*(.*)", line)
            if m:
                n_loads += 1
                touched = _vregs(m.group(3)) & set(pending)
                if touched:
                    bad.append((no, line, sorted(touched)))
                for r in range(int(m.group(1)), int(m.group(2)) + 1):
                    pending[r] = no
                continue
            if line.startswith("s_waitcnt") and "vmcnt" in line:
                pending.clear()       # the naming wait: everything requested before it is retired
                continue
        if pending:
            touched = _vregs(line) & set(pending)
            if touched:
                bad.append((no, line, sorted(touched)))
    return n_loads, bad


def main():
    n, bad = check_register_fed_loads(device_assembly())
    print(f"{n} assembly loads with register destinations, {len(bad)} instructions inside a request-to-retire window touch them")
    for no, line, regs in bad[:20]:
        print(f"  line {no}: {line}   (v{regs})")
    sys.exit(1 if bad or n == 0 else 0)


if __name__ == "__main__":
    main()
