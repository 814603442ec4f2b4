"""The grouped-GEMM kernels read their MFMA operands from LDS with assembly statements (so that the compiler does
not order them behind every outstanding direct global->LDS load).  Such a read delivers asynchronously; the kernels
name the destination registers as operands of the wait that follows, so the compiler must keep them untouched until
then.  This test compiles the kernels to assembly and checks exactly that, instruction by instruction: between an
assembly LDS read and the next wait for the LDS counter, nothing reads, copies, spills or overwrites its destination
registers (CPU only: hipcc cross-compiles without a GPU)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_02317_amd", "csrc")


def _regs(text):
    regs = [int(x) for x in re.findall(r"\bv(\d+)\b", text)]
    for a, b in re.findall(r"v\[(\d+):(\d+)\]", text):
        regs += list(range(int(a), int(b) + 1))
    return regs


def scan_kernel(lines):
    """-> list of (line number, instruction, what) for every touch of a pending destination.
    LDS reads of a wave complete in order: a wait for the counter to drop to N retires all but the last N reads."""
    pending, bad, in_asm, order = {}, [], False, []          # order: destination register lists of the reads in flight
    vm_order = []                                            # the same for vector-memory instructions (most have no tracked destination)
    for i, line in enumerate(lines):
        if "#ASMSTART" in line:
            in_asm = True
            continue
        if "#ASMEND" in line:
            in_asm = False
            continue
        st = line.strip()
        m = in_asm and re.match(r"ds_read_b(?:64_tr_b16|128) v\[(\d+):(\d+)\]", st)
        if m:
            dst = list(range(int(m.group(1)), int(m.group(2)) + 1))
            for r in dst:
                if r in pending:
                    bad.append((i, st, "overwrites a pending destination"))
                pending[r] = i
            order.append(dst)
            continue
        # a scale word requested by an assembly statement: pending until a wait for the vector-memory counter retires it
        # (vector-memory instructions complete in order; every one of them counts)
        m = in_asm and re.match(r"global_load_dword v(\d+),", st)
        if m:
            r = int(m.group(1))
            if r in pending:
                bad.append((i, st, "overwrites a pending destination"))
            pending[r] = i
            vm_order.append([r])
            continue
        if re.match(r"(global|scratch|buffer|flat)_(load|store|atomic)", st):
            if any(r in pending for r in _regs(st)):
                bad.append((i, st, "touches a pending destination"))
            vm_order.append([])
            continue
        w = st.startswith("s_waitcnt") and re.search(r"vmcnt\((\d+)\)", st)
        if w:
            keep = int(w.group(1))
            while len(vm_order) > keep:
                for r in vm_order.pop(0):
                    pending.pop(r, None)
        w = st.startswith("s_waitcnt") and re.search(r"lgkmcnt\((\d+)\)", st)
        if w:
            keep = int(w.group(1))
            while len(order) > keep:
                for r in order.pop(0):
                    pending.pop(r, None)
            continue
        if re.match(r"s_branch\b", st) or st.startswith("s_endpgm"):
            pending, order, vm_order = {}, [], []      # what follows is reached from elsewhere
            continue
        if not st or st[0] in ";." or st.startswith("s_") or st.endswith(":"):
            continue
        if any(r in pending for r in _regs(st)):
            bad.append((i, st, "touches a pending destination"))
    return bad


def test_scanner_sees_a_planted_hazard():
    good = ["\t;;#ASMSTART", "\tds_read_b128 v[10:13], v1 offset:64", "\t;;#ASMEND", "\tv_add_u32_e32 v2, v3, v4",
            "\ts_waitcnt lgkmcnt(0)", "\tv_mov_b32_e32 v5, v10"]
    assert scan_kernel(good) == []
    copied = good[:3] + ["\tv_mov_b32_e32 v20, v11"] + good[3:]
    assert len(scan_kernel(copied)) == 1
    spilled = good[:3] + ["\tscratch_store_dwordx4 off, v[10:13], off offset:16"] + good[3:]
    assert len(scan_kernel(spilled)) == 1
    clobbered = good[:3] + ["\t;;#ASMSTART", "\tds_read_b64_tr_b16 v[12:13], v1", "\t;;#ASMEND"] + good[3:]
    assert len(scan_kernel(clobbered)) == 2
    # partial waits: two reads in flight, a wait for all but one retires the first only
    two = ["\t;;#ASMSTART", "\tds_read_b128 v[10:13], v1", "\t;;#ASMEND", "\t;;#ASMSTART", "\tds_read_b128 v[14:17], v1 offset:16", "\t;;#ASMEND",
           "\t;;#ASMSTART", "\ts_waitcnt lgkmcnt(1)", "\t;;#ASMEND"]
    assert scan_kernel(two + ["\tv_mov_b32_e32 v5, v10"]) == []
    assert len(scan_kernel(two + ["\tv_mov_b32_e32 v5, v14"])) == 1
    # a requested word followed by two younger loads: a wait for all but two retires it, a wait for all but three does not
    word = ["\t;;#ASMSTART", "\tglobal_load_dword v7, v1, s[2:3]", "\t;;#ASMEND", "\tglobal_load_lds_dwordx4 v[2:3], off",
            "\tglobal_load_lds_dwordx4 v[4:5], off"]
    assert scan_kernel(word + ["\ts_waitcnt vmcnt(2)", "\tv_lshrrev_b32_e32 v8, v9, v7"]) == []
    assert len(scan_kernel(word + ["\ts_waitcnt vmcnt(3)", "\tv_lshrrev_b32_e32 v8, v9, v7"])) == 1


def test_no_instruction_touches_a_pending_lds_read(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    from paper_2508_02317_amd.build import HIPCC_FLAGS
    out = str(tmp_path / "gemm_bf16.s")
    flags = [f for f in HIPCC_FLAGS if f != "-fPIC"]
    res = subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", os.path.join(CSRC, "gemm_bf16.hip"), "-o", out],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    text = open(out).read()
    kernels = re.split(r"\n(?=_ZN3moe[^\n]*:\s*;\s*@)", text)
    checked = 0
    for k in kernels:
        name = k.split(":")[0]
        if "row_grouped_kernel" not in name and "wgrad_kernel" not in name and "mx8_row_kernel" not in name:
            continue
        lines = k.split("\n")
        n_reads = sum(1 for l in lines if re.match(r"\s*ds_read_b(?:64_tr_b16|128) ", l))
        assert n_reads > 0, name
        bad = scan_kernel(lines)
        assert not bad, "%s: %s" % (name, bad[:5])
        checked += 1
    assert checked >= 13
