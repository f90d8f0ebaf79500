"""Guard against a code-generation fault met while writing the kernels: for a
clamped 64-bit length that also fed a branch, hipcc emitted an ``s_cselect``
after the branch whose condition code had been overwritten by an unrelated
``s_addc_u32`` -- a short unit was processed as a full one.  The kernels were
rewritten so that the pattern does not arise; this test compiles them to gfx950
assembly (no GPU needed) and checks that every scalar select / SCC branch reads
a condition code produced by a compare or a mask operation."""
import os
import re
import subprocess

from paper_1811_03619_amd import buildlib

SCC_WRITERS = re.compile(
    r"^\s*(s_cmp\w*|s_and\w*|s_or\w*|s_xor\w*|s_andn2\w*|s_orn2\w*|s_nand\w*|s_nor\w*|s_xnor\w*|s_add\w*|s_sub\w*|"
    r"s_lshl\w*|s_lshr\w*|s_ashr\w*|s_bfe\w*|s_min\w*|s_max\w*|s_abs\w*|s_not\w*|s_bitcmp\w*|s_bcnt\w*|s_wqm\w*|"
    r"s_quadmask\w*|s_absdiff\w*)\s")
GOOD = re.compile(r"s_cmp|s_and|s_or|s_xor|s_andn2|s_orn2|s_bitcmp|label")


def test_scalar_selects_read_a_fresh_condition_code(tmp_path):
    asm = tmp_path / "kernels.s"
    flags = [f for f in buildlib.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + ["-I", buildlib.INCLUDE, "-S", "--cuda-device-only",
                                                                       os.path.join(buildlib.CSRC, "pipesgd_kernels.hip"),
                                                                       "-o", str(asm)]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    last, kernel, uses, bad = None, None, 0, []
    for i, line in enumerate(asm.read_text().split("\n")):
        if re.match(r"^_Z\w+:", line):
            kernel, last = line.split(":")[0], None
        if line.startswith(".LBB"):
            last = "label"
        m = SCC_WRITERS.match(line)
        if m:
            last = m.group(1)
        if re.match(r"^\s*(s_cselect|s_cbranch_scc)", line):
            uses += 1
            if last is not None and not GOOD.match(last):
                bad.append((kernel, i, last, line.strip()))
    assert uses > 100, "the scan found no scalar selects at all: the pattern list is out of date"
    assert not bad, bad[:5]
