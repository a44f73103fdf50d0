"""A check of the compiler's output, not of the library's results.

hipcc (ROCm 7.2, gfx950) has been seen to miscompile two back-to-back uniform 64-bit compare-and-selects:
both compares are vector compares into vcc, the first is copied to the scalar condition code
(s_and_b64 ..., vcc, exec) for its s_cselect, and the second s_cselect then reuses that stale condition
instead of its own compare.  The tier planner's 64-way search hit it (its source now keeps the round's count
in a vector register); this test compiles every kernel source to assembly and looks for the same sequence,
so that new code that runs into it fails here and not in a rare data-dependent case on the GPU."""
import glob
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2301_02959_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# scalar instructions that leave the condition code alone
KEEPS_SCC = re.compile(r"s_(mov|cmov|load|buffer_load|waitcnt|branch|cbranch|cselect|nop|endpgm|barrier|sleep|setprio|"
                       r"getreg|setreg|getpc|setpc|swappc|movk|mul_i32|mul_hi|pack|sendmsg|trap|code_end)")


def stale_condition_selects(asm: str):
    """(line number, text) of every s_cselect that reuses a vcc -> SCC copy which an earlier group of selects
    has already consumed, after vcc has been written again (the second compare's selects running on the first
    compare's condition).  One group of selects right after the copy is the compiler's ordinary scheduling even
    if the next vector compare has been hoisted above it: the condition code still holds the first compare."""
    hits = []
    from_vcc = False          # SCC currently holds a copy of vcc
    vcc_rewritten = False     # ... and a later vector compare has replaced vcc since
    selecting = False         # the previous instruction was an s_cselect on this copy
    consumed = False          # ... a group of selects on this copy has ended
    for no, line in enumerate(asm.split("\n"), 1):
        text = line.strip()
        if not text or text.startswith(";") or text.startswith("."):
            if re.match(r"^\.?[\w$]+:", text):
                from_vcc = vcc_rewritten = selecting = consumed = False
            continue
        if re.match(r"^[\w$.]+:", text):                       # a label: unknown predecessor
            from_vcc = vcc_rewritten = selecting = consumed = False
            continue
        op = text.split()[0]
        if op.startswith("s_cselect"):
            if from_vcc and vcc_rewritten and consumed:
                hits.append((no, text))
            selecting = from_vcc
            continue
        if selecting:
            consumed, selecting = True, False
        if op.startswith("v_cmp") and (op.endswith("_e32") or re.search(r"\bvcc\b", text.split(",")[0])):
            if from_vcc:
                vcc_rewritten = True
            continue
        if op.startswith("s_") and not KEEPS_SCC.match(op):
            from_vcc = bool(re.match(r"s_and_b64\s+\S+\s+(vcc, exec|exec, vcc)$", text))
            vcc_rewritten = consumed = False
    return hits


def test_scanner_sees_the_known_sequence():
    bad = """
	v_cmp_lt_i64_e32 vcc, s[12:13], v[6:7]
	s_and_b64 s[14:15], vcc, exec
	s_cselect_b32 s5, s13, s5
	s_cselect_b32 s4, s12, s4
	v_mov_b64_e32 v[6:7], s[4:5]
	v_cmp_lt_i64_e32 vcc, s[8:9], v[6:7]
	s_cselect_b32 s9, s9, s5
	s_cselect_b32 s8, s8, s4
"""
    good = bad.replace("\ts_cselect_b32 s9, s9, s5", "\ts_and_b64 s[14:15], vcc, exec\n\ts_cselect_b32 s9, s9, s5")
    assert [n for n, _ in stale_condition_selects(bad)] == [8, 9]
    assert stale_condition_selects(good) == []
    # the second compare hoisted above the first compare's selects: each pair still runs on its own condition
    hoisted = """
	v_cmp_gt_i64_e32 vcc, s[6:7], v[34:35]
	s_and_b64 s[22:23], vcc, exec
	v_cmp_lt_i64_e32 vcc, s[20:21], v[36:37]
	s_cselect_b32 s49, s7, s27
	s_cselect_b32 s48, s6, s26
	s_and_b64 s[6:7], vcc, exec
	s_cselect_b32 s43, s21, s9
	s_cselect_b32 s42, s20, s8
"""
    assert stale_condition_selects(hoisted) == []
    # ... and without the second copy the second pair is stale
    assert [n for n, _ in stale_condition_selects(hoisted.replace("\ts_and_b64 s[6:7], vcc, exec\n", "\tv_mov_b32_e32 v1, s48\n"))] == [8, 9]


@pytest.mark.skipif(shutil.which(HIPCC) is None and not os.path.exists(HIPCC), reason="hipcc not found")
def test_no_kernel_selects_on_a_stale_condition(tmp_path):
    from paper_2301_02959_amd.build import FLAGS
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    procs = []
    for src in sorted(glob.glob(os.path.join(CSRC, "*.hip"))):
        out = tmp_path / (os.path.basename(src) + ".s")
        cmd = [HIPCC, *flags, "--cuda-device-only", "-S", src, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", str(out)]
        procs.append((src, out, subprocess.Popen(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.PIPE, text=True)))
    for src, out, p in procs:
        _, err = p.communicate()
        assert p.returncode == 0, err[-2000:]
        hits = stale_condition_selects(out.read_text())
        assert not hits, f"{os.path.basename(src)}: s_cselect on a stale condition code at assembly lines {hits[:4]}"
