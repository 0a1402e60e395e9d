"""Host-side check of the generated gfx950 code around the hand-written inline assembly.

The LDS-DMA helper of the prefill kernel narrows EXEC with scalar logic instructions (s_and_b64,
s_andn2_b64; formerly s_not_b64), which also write SCC.
If the asm statement did not declare that, the compiler could keep the carry of a 64-bit
address addition alive across the block (s_add_u32 before it, s_addc_u32 after it); the
address then comes out 4 GiB off and the copy faults.  This test compiles every file whose kernels
contain the helper to assembly and looks for any SCC reader that follows an inline-asm block without an SCC
writer in between.  (The toolchain cross-compiles; no GPU is needed.)"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2410_01228_amd", "csrc")
ASM_HOME = os.path.join(CSRC, "cs_prefill_impl.h")            # where the inline assembly is written
USERS = ["cs_prefill.hip", "cs_mixed.hip"]                     # the files whose kernels contain it

SCC_READER = re.compile(r"^(s_cbranch_scc[01]|s_addc_u32|s_subb_u32|s_cselect_b(32|64)|s_cmov_b(32|64))\b")
# scalar instructions that leave SCC alone; every other s_* instruction is taken to write it
SCC_NEUTRAL = re.compile(r"^(s_mov|s_movk|s_cmov|s_cselect|s_mul_|s_load|s_buffer|s_nop|s_waitcnt|s_barrier|s_branch|"
                         r"s_cbranch|s_endpgm|s_getpc|s_setpc|s_swappc|s_setprio|s_sleep|s_sendmsg|s_setreg|s_getreg|"
                         r"s_brev|s_sext|s_pack|s_bfm|s_ff1|s_ff0|s_flbit|s_bitset|s_dcache|s_icache|s_trap|s_ttrace|"
                         r"s_memtime|s_memrealtime|s_sethalt|s_setvskip|s_set_gpr_idx|s_inst_prefetch)")


def scc_reads_after_asm(asm_text):
    """(line number, instruction) of every SCC reader reached from the end of an inline-asm
    block that writes SCC without passing an SCC writer (labels are walked through: the
    fall-through path is the one the scheduler created)."""
    lines = asm_text.split("\n")
    found = []
    i = 0
    while i < len(lines):
        if "ASMSTART" in lines[i]:
            j = i
            body = []
            while "ASMEND" not in lines[j]:
                body.append(lines[j].strip())
                j += 1
            if any(b.startswith(("s_not_b64", "s_and_b64", "s_andn2_b64")) for b in body):
                k = j + 1
                while k < len(lines):
                    t = lines[k].strip()
                    k += 1
                    if not t or t.startswith(";") or t.startswith(".") or t.endswith(":"):
                        continue
                    op = t.split()[0]
                    if SCC_READER.match(op):
                        found.append((k, t))
                        break
                    if op.startswith("s_") and not SCC_NEUTRAL.match(op):
                        break                                   # SCC rewritten: whatever the asm left is dead
                    if op in ("s_endpgm", "s_branch") or "ASMSTART" in t:
                        break
            i = j
        i += 1
    return found


def test_scanner_sees_a_planted_hazard():
    bad = """
	s_add_u32 s66, s22, s38
	;;#ASMSTART
	s_mov_b32 m0, s47
	s_not_b64 exec, exec
	;;#ASMEND
	s_addc_u32 s67, s23, s39
"""
    good = bad.replace("s_addc_u32 s67, s23, s39", "s_add_i32 s7, s60, s21\n\ts_addc_u32 s67, s23, s39")
    assert len(scc_reads_after_asm(bad)) == 1
    assert scc_reads_after_asm(good) == []
    bad2 = bad.replace("s_not_b64 exec, exec", "s_andn2_b64 exec, s[4:5], s[6:7]")
    assert len(scc_reads_after_asm(bad2)) == 1


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
@pytest.mark.parametrize("src", USERS)
def test_no_scc_value_lives_across_the_dma_asm(tmp_path, src):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    out = tmp_path / (src + ".s")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(CSRC, src)]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = out.read_text()
    assert text.count("global_load_lds_dwordx4") > 50, "the DMA blocks are gone from the kernel?"
    hazards = scc_reads_after_asm(text)
    assert hazards == [], "SCC read after an inline-asm block that rewrote it: %r" % hazards[:5]
    # and the statement says so itself
    assert '"scc"' in open(ASM_HOME).read()
    # EXEC is put back as it was found, never forced to all lanes
    assert "s_mov_b64 exec, -1" not in text and "s_andn2_b64 exec" in text
