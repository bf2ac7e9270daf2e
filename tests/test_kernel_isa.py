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


# ------------------------------------------------------------------------------------------------ attention
VMEM = ("global_load", "global_store", "global_atomic", "buffer_", "scratch_", "flat_")


def scan_attention(text, kernel_filter="attn_bf16_kernel"):
    """Walks every bf16 attention kernel in program order and checks what its hand-written synchronisation assumes:

    pages      a page moves with eight direct-to-LDS loads issued back to back; the producer's waits (`s_waitcnt
               vmcnt(8)`: everything but the youngest page has landed) count exactly those, so no other
               vector-memory instruction may sit inside a run of them, and every run is a whole number of pages;
    hand-over  a work item publishes its state with device-coherent stores (sc1), waits until all of them are
               acknowledged (`s_waitcnt vmcnt(0)`), passes a workgroup barrier, and only then bumps the arrival
               counter (the one returning atomic add); whoever arrives last reads the states with device-coherent
               loads (sc1).
    Returns (kernels, page runs, violations)."""
    violations, n_kern, n_runs = [], 0, 0
    kernels, cur = [], None
    for line in text.split("\n"):
        m = re.match(r"^(_Z\S+):", line)
        if m:
            cur = [] if kernel_filter in m.group(1) else None
            if cur is not None:
                kernels.append((m.group(1), cur))
            continue
        t = line.strip()
        if cur is None or not t or t[0] in ";.":
            continue
        cur.append(t)
    for name, ins in kernels:
        n_kern += 1
        short = re.search(r"attn_bf16_kernelILi(\d)ELb(\d)", name)
        tag = f"attn<{short.group(1)},{short.group(2)}>" if short else name[:40]
        # ---- pages
        i = 0
        saw_wait8 = 0
        while i < len(ins):
            if ins[i].startswith("s_waitcnt") and "vmcnt(8)" in ins[i]:
                saw_wait8 += 1
            if ins[i].startswith("global_load_lds_dwordx4"):
                run, j = 0, i
                while j < len(ins) and not (ins[j].startswith("s_waitcnt") and "vmcnt" in ins[j]) and not ins[j].startswith("s_barrier") \
                        and not ins[j].startswith("s_cbranch") and not ins[j].startswith("s_branch"):
                    if ins[j].startswith("global_load_lds_dwordx4"):
                        run += 1
                    elif ins[j].startswith(VMEM):
                        violations.append(f"{tag}: `{ins[j]}` inside a run of page loads")
                    j += 1
                if run % 8:
                    violations.append(f"{tag}: a run of {run} page loads is not a whole number of pages")
                n_runs += 1
                i = j
                continue
            i += 1
        if saw_wait8 < 2:
            violations.append(f"{tag}: the producer's s_waitcnt vmcnt(8) are missing")
        # ---- hand-over
        adds = [k for k, t in enumerate(ins) if t.startswith("global_atomic_add") and " sc0" in t + " "]
        if len(adds) != 1:
            violations.append(f"{tag}: expected one returning atomic add (the arrival counter), found {len(adds)}")
            continue
        a = adds[0]
        b = max((k for k in range(a) if ins[k].startswith("s_barrier")), default=-1)
        if b < 0:
            violations.append(f"{tag}: no workgroup barrier before the arrival counter")
            continue
        # the stores of the state: the block of sc1 stores that ends at the wait before that barrier
        w = max((k for k in range(b) if ins[k].startswith("s_waitcnt") and "vmcnt(0)" in ins[k]), default=-1)
        stores = [k for k in range(max(0, w - 200), b) if ins[k].startswith("global_store")]
        if w < 0 or not stores:
            violations.append(f"{tag}: no acknowledged stores before the barrier that precedes the arrival counter")
        else:
            if any(k > w for k in stores):
                violations.append(f"{tag}: a store of the state is issued after the wait for the acknowledgements")
            state = [k for k in stores if k > w - 60]
            if len(state) < 10:
                violations.append(f"{tag}: only {len(state)} stores of the state found before the wait")
            for k in state:
                if " sc1" not in ins[k] + " ":
                    violations.append(f"{tag}: `{ins[k]}` publishes state without device coherence (sc1)")
        nxt = next((k for k in range(a + 1, len(ins)) if ins[k].startswith("s_barrier")), len(ins))
        nxt2 = next((k for k in range(nxt + 1, len(ins)) if ins[k].startswith("s_barrier")), len(ins))
        merge_loads = [k for k in range(nxt, nxt2) if ins[k].startswith("global_load_dword")]
        if len(merge_loads) < 10:
            violations.append(f"{tag}: the merge's loads of the stored states were not found ({len(merge_loads)})")
        for k in merge_loads:
            if " sc1" not in ins[k] + " ":
                violations.append(f"{tag}: `{ins[k]}` reads a stored state without device coherence (sc1)")
    return n_kern, n_runs, violations


def test_attention_scan_finds_planted_mistakes():
    good = """_Z16attn_bf16_kernelILi1ELb0EEv:
	s_waitcnt vmcnt(8)
	s_waitcnt vmcnt(8)
""" + "\tglobal_load_lds_dwordx4 v[6:7], off\n" * 8 + "\ts_barrier\n" + \
        "\tglobal_store_dwordx2 v[34:35], v[2:3], off sc1\n" * 12 + """	s_waitcnt vmcnt(0) expcnt(0) lgkmcnt(0)
	s_barrier
	global_atomic_add v35, v35, v36, s[10:11] sc0
	s_barrier
""" + "\tglobal_load_dwordx2 v[34:35], v[102:103], off sc1\n" * 12 + "\ts_barrier\n\ts_endpgm\n"
    assert scan_attention(good)[2] == []
    assert any("whole number" in v for v in scan_attention(good.replace("\tglobal_load_lds_dwordx4 v[6:7], off\n", "", 1))[2])
    assert any("inside a run" in v for v in scan_attention(good.replace(
        "\tglobal_load_lds_dwordx4 v[6:7], off\n", "\tglobal_load_lds_dwordx4 v[6:7], off\n\tglobal_load_dword v1, v[2:3], off\n", 1))[2])
    assert any("without device coherence" in v for v in scan_attention(good.replace("v[2:3], off sc1", "v[2:3], off", 1))[2])
    assert any("without device coherence" in v for v in scan_attention(good.replace("v[102:103], off sc1", "v[102:103], off", 1))[2])
    assert any("acknowledged" in v or "after the wait" in v for v in scan_attention(good.replace("\ts_waitcnt vmcnt(0) expcnt(0) lgkmcnt(0)\n", ""))[2])


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_attention_kernels_keep_their_hand_written_synchronisation():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attention.s")
        flags = [f for f in B.FLAGS if f != "-fPIC"]
        cmd = ["hipcc", *flags, "--cuda-device-only", "-S", os.path.join(B.CSRC, "attention.hip"), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(out).read()
    n_kern, n_runs, bad = scan_attention(text)
    assert n_kern == 10 and n_runs >= 3 * n_kern, (n_kern, n_runs)
    assert not bad, "\n".join(bad[:20])
