"""Build-time guard on the generated gfx950 code of the kernels.

One build of the vector kernel read the scalar condition code in an s_cselect whose producer the
compiler had dropped (a uniform 64-bit compare feeding both a branch and a select), which made short
last tiles run at full length.  The source no longer has that shape; this test compiles the kernels to
assembly and checks that every SCC consumer has a comparison or logic producer in its own basic block."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = "/opt/rocm/bin/hipcc"

PRODUCER = re.compile(r"^\s*(s_cmp|s_cmpk|s_bitcmp|s_and_|s_or_|s_andn2|s_orn2|s_xor|s_xnor|s_nand|s_nor|s_not|"
                      r"s_add_|s_addc|s_sub_|s_subb|s_lshl|s_lshr|s_ashr|s_bfe|s_abs|s_min|s_max|s_absdiff|s_bcnt|"
                      r"s_ff|s_flbit|s_wqm|s_quadmask|s_addk)")
ARITH = re.compile(r"(s_addc|s_subb|s_lshl|s_lshr|s_bfe|s_sub_|s_add_)")


def scc_findings(asm_text):
    lines = asm_text.split("\n")
    found = []
    for i, l in enumerate(lines):
        if not re.match(r"^\s*(s_cselect|s_cbranch_scc)", l):
            continue
        prod = None
        for j in range(i - 1, -1, -1):
            t = lines[j]
            if re.match(r"^\.LBB", t) or re.match(r"^_Z", t):
                prod = "LABEL"
                break
            if PRODUCER.match(t):
                prod = t.strip()
                break
        carry_use = "s_cselect_b64" in l and "-1" in l        # carry/borrow turned into a mask: intended
        if prod == "LABEL" or (prod and ARITH.match(prod) and not carry_use):
            found.append((i + 1, l.strip(), prod))
    return found


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_no_scc_consumer_without_producer(tmp_path):
    out = tmp_path / "kernels.s"
    from paper_2505_23072_amd.build import DEVICE_FLAGS
    subprocess.check_call([HIPCC] + DEVICE_FLAGS + ["-S", "--cuda-device-only", "-o", str(out),
                                                    os.path.join(ROOT, "paper_2505_23072_amd", "csrc", "kernels.hip")],
                          stderr=subprocess.DEVNULL)
    text = out.read_text()
    assert "materialize_vec" in text and "global_load_dwordx4" in text
    assert "flat_load" not in text and "flat_store" not in text, "generic-address accesses crept back in"
    assert "scratch_" not in text, "register spills"
    assert scc_findings(text) == []
    # the conversion instructions depend on the kernels' floating-point mode: round to nearest even,
    # denormals kept for every width (a flush-to-zero or fast-math build flag would change these)
    n_kernels = len(re.findall(r"^\s*\.amdhsa_kernel ", text, flags=re.M))
    assert n_kernels >= 28
    for directive, value in ((".amdhsa_float_round_mode_32", 0), (".amdhsa_float_round_mode_16_64", 0),
                             (".amdhsa_float_denorm_mode_32", 3), (".amdhsa_float_denorm_mode_16_64", 3)):
        found = re.findall(rf"^\s*{re.escape(directive)}\s+(\d+)", text, flags=re.M)
        assert len(found) == n_kernels and all(int(v) == value for v in found), (directive, sorted(set(found)))


def test_checker_catches_the_known_bad_shape():
    bad = "\n".join([".LBB0_9:", "\ts_add_u32 s8, s0, s6", "\ts_addc_u32 s9, s1, s7",
                     "\tv_cmp_lt_u64_e32 vcc, s[2:3], v[2:3]", "\ts_cbranch_vccz .LBB0_33",
                     "\ts_cselect_b32 s17, s2, 0x1000"])
    assert len(scc_findings(bad)) == 1
    good = bad.replace("\ts_cbranch_vccz .LBB0_33", "\ts_and_b64 s[2:3], vcc, exec")
    assert scc_findings(good) == []
