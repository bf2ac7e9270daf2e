"""Static check of the projection kernel's machine code (no GPU needed: hipcc cross-compiles).

The kernel issues its weight loads from inline assembly and waits for them with hand-counted `s_waitcnt vmcnt`
(csrc/gemm.hip).  The compiler sees such a load as complete when it is issued, so nothing stops it from moving or
reusing the destination registers while the data is still on its way -- which it does, for instance, when a branch
separates a load from its wait.  The results are then wrong without any error.  This test compiles gemm.hip to
assembly with the library's own flags and walks every bf16 projection kernel in program order: loads retire in
order, `s_waitcnt vmcnt(N)` leaves the N youngest in flight, and between a load and the wait that covers it no
instruction may name its destination registers.
"""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

from paper_2506_09397_amd import build as B


def _regs(tok):
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", tok)
    return {int(m.group(1))} if m else set()


def scan(text, kernel_filter):
    """Returns (kernels scanned, hand-issued register loads seen, list of violations)."""
    violations, n_kern, n_loads = [], 0, 0
    active, inflight, in_asm = False, [], False
    for ln, line in enumerate(text.split("\n"), 1):
        m = re.match(r"^(_Z\S+):", line)
        if m:
            active = kernel_filter in m.group(1)
            n_kern += active
            inflight = []
            continue
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not active or not t or t[0] in ";.":
            continue
        op = t.split()[0]
        args = [a.strip() for a in t[len(op):].split(",")]
        if op == "s_endpgm":
            inflight = []
            continue
        if op.startswith("s_waitcnt"):
            m = re.search(r"vmcnt\((\d+)\)", t)
            if m:
                n = int(m.group(1))
                inflight = inflight[len(inflight) - n:] if 0 < n < len(inflight) else ([] if n == 0 else inflight)
            continue
        if op.startswith("global_load_lds") or op.startswith("global_store") or op.startswith("global_atomic"):
            inflight.append(set())          # counted by vmcnt, no register destination
            continue
        touched = set()
        for a in args:
            for tok in re.findall(r"v\[\d+:\d+\]|v\d+", a):
                touched |= _regs(tok)
        for dest in inflight:
            if dest & touched:
                violations.append(f"line {ln}: `{t}` names v{sorted(dest & touched)} while a load into them is in flight")
        if op.startswith("global_load"):
            dest = _regs(args[0])
            inflight.append(dest if in_asm else set())   # compiler-issued loads are the compiler's to track
            n_loads += in_asm
    return n_kern, n_loads, violations


def test_scan_finds_a_planted_copy():
    text = """_Z4demov:
	;;#ASMSTART
	global_load_dwordx4 v[38:41], v[66:67], off
	;;#ASMEND
	v_mov_b64_e32 v[62:63], v[40:41]
	;;#ASMSTART
	s_waitcnt vmcnt(0)
	;;#ASMEND
	v_mov_b64_e32 v[60:61], v[38:39]
	s_endpgm
"""
    n_kern, n_loads, bad = scan(text, "demo")
    assert (n_kern, n_loads) == (1, 1) and len(bad) == 1 and "v_mov_b64_e32 v[62:63]" in bad[0]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_no_instruction_touches_a_register_with_a_load_in_flight():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm.s")
        flags = [f for f in B.FLAGS if f != "-fPIC"]
        cmd = ["hipcc", *flags, "--cuda-device-only", "-S", os.path.join(B.CSRC, "gemm.hip"), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(out).read()
    n_kern, n_loads, bad = scan(text, "gemm_bf16_kernel")
    assert n_kern >= 15 and n_loads > 100 * n_kern // 10, (n_kern, n_loads)
    assert not bad, "\n".join(bad[:20])
