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
    """-> list of (line number, instruction, what) for every touch of a pending destination."""
    pending, bad, in_asm = {}, [], False
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
            for r in range(int(m.group(1)), int(m.group(2)) + 1):
                if r in pending:
                    bad.append((i, st, "overwrites a pending destination"))
                pending[r] = i
            continue
        if st.startswith("s_waitcnt") and "lgkmcnt(0)" in st:
            pending = {}
            continue
        if re.match(r"s_branch\b", st) or st.startswith("s_endpgm"):
            pending = {}                      # what follows is reached from elsewhere
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
        if "row_grouped_kernel" not in name and "wgrad_kernel" not in name:
            continue
        lines = k.split("\n")
        n_reads = sum(1 for l in lines if re.match(r"\s*ds_read_b(?:64_tr_b16|128) ", l))
        assert n_reads > 0, name
        bad = scan_kernel(lines)
        assert not bad, "%s: %s" % (name, bad[:5])
        checked += 1
    assert checked >= 10
