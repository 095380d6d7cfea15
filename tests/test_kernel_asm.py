"""A property of the generated code that the source relies on and cannot express (CPU only: hipcc cross-compiles).

attn_fwd64 reads every V fragment with two transposed LDS reads whose results land asynchronously; the source
joins the two halves into the register quadruple of an MFMA operand right at the reads.  That is only correct if
the compiler makes the reads write the quadruple's halves directly: a register copy between a read and the
wait for it would copy stale data.  The check: in the compiled kernel every pair of consecutive transposed reads
fills two adjacent register pairs, and that quadruple is read by an MFMA as it stands."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")
def test_v_fragments_are_read_into_the_mfma_operand_registers():
    from paper_2409_09086_amd.build import CSRC, FLAGS
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "attn_mfma64.s")
        subprocess.run(["hipcc", *[f for f in FLAGS if f != "-fPIC"], "-I" + os.path.join(ROOT, "include"), "-S",
                        "--cuda-device-only", os.path.join(CSRC, "attn_mfma64.hip"), "-o", asm],
                       check=True, capture_output=True)
        lines = open(asm).read().splitlines()
    reads = [int(m.group(1)) for l in lines for m in [re.search(r"ds_read_b64_tr_b16 v\[(\d+):(\d+)\]", l)] if m]
    assert len(reads) >= 64 and len(reads) % 2 == 0, len(reads)
    quads = set()
    for lo, hi in zip(reads[0::2], reads[1::2]):
        assert hi == lo + 2, "the two halves of a V fragment do not fill one register quadruple: v%d, v%d" % (lo, hi)
        quads.add((lo, lo + 3))
    operands = set()
    for l in lines:
        m = re.search(r"v_mfma_f32_32x32x16_bf16 a\[\d+:\d+\], v\[(\d+):(\d+)\], v\[", l)
        if m:
            operands.add((int(m.group(1)), int(m.group(2))))
    assert operands, "no O += V^T P^T product found"
    missing = sorted(quads - operands)
    assert not missing, "V fragments that no MFMA reads from the registers they were read into: %s" % missing
