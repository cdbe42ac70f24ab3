"""The prefill main kernel and the large-batch router write their MFMAs as inline
assembly with the accumulators in AccVGPRs.  The compiler does not look inside an assembly statement, so its
hazard recogniser does not know that those statements are MFMAs: a register copy that IT places right behind one
(to resolve a phi, to make room) would read an accumulator while the matrix core is still writing it, with no
error.  This test compiles the kernels to assembly (no GPU) and checks, in every kernel with assembly MFMAs, that
 * nothing is spilled to scratch memory (a reload waits for every direct-to-LDS load in flight), and
 * every AccVGPR access the compiler emitted itself (outside the assembly statements) keeps its distance from the
   last MFMA that wrote that register, and every such write from the last MFMA that read the register as its
   addend: at least MIN_GAP other instructions, or s_nops worth as much; and no MFMA reads an AccVGPR that the
   compiler wrote fewer than MIN_GAP_AFTER_WRITE instructions before.
The scan follows the listing top to bottom; it does not follow branches, so a copy at a loop's head is checked
against the MFMAs listed above it, not against those at the loop's end.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2410_09687_amd import build as B

MIN_GAP = 6          # instructions (4 cycles each at the least) between an MFMA of 4 passes and a read of its result
MIN_GAP_AFTER_WRITE = 3
KERNELS = {"linear_stream.hip": "linear_stream_kernel", "route.hip": "route_stream4_kernel"}


def _device_asm(src):
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        flags = [f for f in B.FLAGS if f != "-fPIC"]
        r = subprocess.run([B.HIPCC, *flags, "-S", "--cuda-device-only", "-o", out, os.path.join(B.CSRC, src)],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return open(out).read()


def _kernel_bodies(asm, name):
    """(symbol, lines) of every kernel whose mangled name contains `name`"""
    out, cur, sym = [], None, None
    for line in asm.split("\n"):
        m = re.match(r"^(_Z\w+):", line)
        if m and name in m.group(1):
            sym, cur = m.group(1), []
        elif cur is not None:
            cur.append(line)
            if "s_endpgm" in line:
                out.append((sym, cur))
                cur = None
    return out


def _regs(tok):
    m = re.match(r"a\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"a(\d+)$", tok)
    return {int(m.group(1))} if m else set()


@pytest.mark.parametrize("src", sorted(KERNELS))
def test_no_scratch_and_no_early_accvgpr_access(src):
    asm = _device_asm(src)
    bodies = _kernel_bodies(asm, KERNELS[src])
    assert bodies, f"no kernel named {KERNELS[src]} in {src}"
    for sym, lines in bodies:
        assert not any(re.search(r"\bscratch_(load|store)", l) for l in lines), f"{sym} spills to scratch"
        in_asm = False
        last_write = {}      # AccVGPR -> instruction count at the MFMA that wrote it last
        last_addend = {}     # AccVGPR -> instruction count at the MFMA that read it last as its addend
        last_copy = {}       # AccVGPR -> instruction count at the compiler-placed instruction that wrote it last
        count = 0            # instructions so far, an s_nop N counted as its N + 1 wait states / 4
        n_mfma = 0
        for line in lines:
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
                continue
            if t.startswith(";;#ASMEND"):
                in_asm = False
                continue
            if not t or t.startswith(";") or t.startswith(".") or t.endswith(":"):
                continue
            op, _, rest = t.partition(" ")
            args = [a.strip() for a in rest.split(",")]
            if op == "s_nop":
                count += (int(args[0]) + 1 + 3) // 4
                continue
            count += 1
            if op.startswith("v_mfma"):
                n_mfma += 1
                for r_ in _regs(args[0]):
                    last_write[r_] = count
                for r_ in _regs(args[3]) if len(args) > 3 else ():
                    last_addend[r_] = count
                    gap = count - last_copy.get(r_, -10 ** 9)
                    assert gap >= MIN_GAP_AFTER_WRITE, f"{sym}: `{t}` reads a{r_} {gap} instructions behind a compiler-placed write"
            elif op.startswith("v_accvgpr") and not in_asm:
                touched = set()
                for a in args:
                    touched |= _regs(a)
                for r_ in touched:
                    gap = count - last_write.get(r_, -10 ** 9)
                    assert gap > MIN_GAP, f"{sym}: compiler-placed `{t}` {gap} instructions behind the MFMA that wrote a{r_}"
                if op in ("v_accvgpr_write_b32", "v_accvgpr_mov_b32"):
                    for r_ in _regs(args[0]):
                        last_copy[r_] = count
                        gap = count - last_addend.get(r_, -10 ** 9)
                        assert gap > MIN_GAP, f"{sym}: compiler-placed `{t}` {gap} instructions behind an MFMA that reads a{r_}"
        assert n_mfma >= 128, f"{sym}: expected the unrolled MFMA blocks, found {n_mfma} MFMAs"


def test_quantised_base_kernel_does_not_spill():
    # its MFMAs are builtins (the compiler sees them and their hazards), but a spill inside its main loop costs
    # the same as in the others: the reload waits for every direct-to-LDS load in flight
    asm = _device_asm("mx.hip")
    bodies = _kernel_bodies(asm, "linear_stream4_kernel")
    assert bodies
    for sym, lines in bodies:
        assert not any(re.search(r"\bscratch_(load|store)", l) for l in lines), f"{sym} spills to scratch"
        assert sum("v_mfma" in l for l in lines) >= 96, f"{sym}: expected the unrolled MFMA blocks"
