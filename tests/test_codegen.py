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
    """(line number, text) of every s_cselect that follows a vcc -> SCC copy after vcc has been written again."""
    hits = []
    from_vcc = False          # SCC currently holds a copy of vcc
    vcc_rewritten = False     # ... and a later vector compare has replaced vcc since
    for no, line in enumerate(asm.split("\n"), 1):
        text = line.strip()
        if not text or text.startswith(";") or text.startswith("."):
            if re.match(r"^\.?[\w$]+:", text):
                from_vcc = vcc_rewritten = False
            continue
        if re.match(r"^[\w$.]+:", text):                       # a label: unknown predecessor
            from_vcc = vcc_rewritten = False
            continue
        op = text.split()[0]
        if op.startswith("s_cselect"):
            if from_vcc and vcc_rewritten:
                hits.append((no, text))
            continue
        if op.startswith("v_cmp") and (op.endswith("_e32") or re.search(r"\bvcc\b", text.split(",")[0])):
            if from_vcc:
                vcc_rewritten = True
            continue
        if op.startswith("s_") and not KEEPS_SCC.match(op):
            from_vcc = bool(re.match(r"s_and_b64\s+\S+\s+(vcc, exec|exec, vcc)$", text))
            vcc_rewritten = False
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
