"""Static check of the compiled bf16 attention kernel's ISA.

The matrix phase of the kernel issues its MFMAs through inline asm, so the compiler does not know
that the registers those statements write are matrix-pipe results: it inserts no wait states if
it decides to read, copy or overwrite one of them with a vector instruction right behind the
MFMA.  The kernel inserts the wait states it needs by hand; this check makes sure the compiler
did not add an access of its own.

Rule checked: a vector register written by a `v_mfma` is not named by any non-MFMA instruction
within WAIT_STATES wait states (one per issued instruction, N + 1 for `s_nop N`) in straight-line
code after it.  (An MFMA that accumulates into the same registers is interlocked by hardware.)
The 32x32x16 bf16 MFMA has 8 passes; the compiler's own rule for it is 11 wait states."""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

from paper_2507_09071_amd import build as _build

WAIT_STATES = 12
KERNELS = ("_ZN2bs17attn_prefill_bf16ILi128EEE", "_ZN2bs17attn_prefill_bf16ILi64EEE")


def compile_to_isa(out_path: str) -> None:
    cmd = [_build.hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-I", os.path.join(_build.ROOT, "include"), "-I", _build.CSRC,
           *os.environ.get("BS_EXTRA_HIPCC_FLAGS", "").split(),
           "--cuda-device-only", "-S", os.path.join(_build.CSRC, "attn_prefill.hip"), "-o", out_path]
    subprocess.run(cmd, check=True, capture_output=True)


def _regs(text: str) -> set:
    out = set()
    for m in re.finditer(r"v\[(\d+):(\d+)\]", text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"(?<![\w\[])v(\d+)\b", text):
        out.add(int(m.group(1)))
    return out


def kernel_instructions(isa: str, symbol_prefix: str) -> list:
    start = isa.index(symbol_prefix)
    end = isa.index("s_endpgm", start)
    ins = []
    for line in isa[start:end].split("\n"):
        t = line.split(";")[0].strip()
        if t and not t.startswith(".") and not t.endswith(":"):
            ins.append(t)
    return ins


def mfma_hazards(ins: list) -> list:
    """List of (mfma, wait states, offending instruction)."""
    found = []
    for a, t in enumerate(ins):
        if not t.startswith("v_mfma"):
            continue
        dst = _regs(t.split(",")[0])
        ws = 0
        for u in ins[a + 1:a + 1 + 4 * WAIT_STATES]:
            if u.startswith(("s_cbranch", "s_branch", "s_barrier", "s_endpgm")):
                break   # the rule is checked in straight-line code only
            if u.startswith("v_mfma"):
                ws += 1
            else:
                if _regs(u) & dst:
                    found.append((t, ws, u))
                m = re.match(r"s_nop (\d+)", u)
                ws += int(m.group(1)) + 1 if m else 1
            if ws >= WAIT_STATES:
                break
    return found


def lds_read_hazards(ins: list) -> list:
    """The operand reads of the matrix phase are asm `ds_read_b128` waited for by hand-counted
    `s_waitcnt lgkmcnt(N)`.  The compiler believes the destination holds the value as soon as
    the asm statement is over; check that nothing names a destination register while its read
    may still be in flight.  LDS reads complete in order: after `lgkmcnt(N)` all but the N
    youngest are done (scalar loads share the counter and only make the wait stricter).
    Straight-line code only: the list of reads in flight is dropped at branches and labels,
    which the kernel never crosses with a read outstanding.  Returns (read, offending
    instruction) pairs."""
    found = []
    inflight = []   # (instruction, destination registers), oldest first
    for t in ins:
        if t.startswith(("s_cbranch", "s_branch", "s_barrier", "s_endpgm")):
            inflight = []
            continue
        m = re.match(r"s_waitcnt .*lgkmcnt\((\d+)\)", t)
        if m:
            n = int(m.group(1))
            inflight = inflight[len(inflight) - n:] if n else []
            continue
        if t.startswith("s_waitcnt") and "lgkmcnt" not in t and "vmcnt" not in t:
            inflight = []   # a bare immediate: treat as a full wait only if it names no counter
            continue
        named = _regs(t)
        for r, dst in inflight:
            if named & dst:
                found.append((r, t))
        if t.startswith("ds_read"):
            inflight.append((t, _regs(t.split(",")[0])))
    return found


def check(isa_path: str | None = None) -> dict:
    """Compile (unless a listing is given) and return {kernel symbol prefix: [hazards]}."""
    if isa_path is None:
        with tempfile.TemporaryDirectory() as d:
            isa_path = os.path.join(d, "attn_prefill.s")
            compile_to_isa(isa_path)
            isa = open(isa_path).read()
    else:
        isa = open(isa_path).read()
    out = {}
    for k in KERNELS:
        ins = kernel_instructions(isa, k)
        out[k] = mfma_hazards(ins) + lds_read_hazards(ins)
    return out


if __name__ == "__main__":
    res = check()
    for k, h in res.items():
        print(k, "hazards:", len(h))
        for item in h[:10]:
            print("  ", *[str(x)[:70] for x in item])
    raise SystemExit(1 if any(res.values()) else 0)
