"""Host-side guard on the generated code of the hot kernels (needs hipcc, no GPU).

The tiled kernel's main loop keeps its DMA queue full only as long as the compiler reloads no
spilled register inside it (it cannot see the inline-assembly loads and drains the queue
before any scratch access it schedules there).  The 128-row, eight-wavefront kernel sits at the
register limit: it spills exactly one register, around the loop and not in it.  A change that
costs it a second spill costs 5 % of the M = 512 benchmark without failing any parity test,
so the scratch sizes are pinned here."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

from paper_2312_08583_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _scratch_sizes(source: str) -> dict:
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        flags = [f for f in B.FLAGS if f not in ("-fPIC",)]
        subprocess.run(["hipcc", *flags, "-S", "--cuda-device-only", os.path.join(B.CSRC, source), "-o", out],
                       check=True, stderr=subprocess.DEVNULL)
        text = open(out).read()
    sizes = {}
    for m in re.finditer(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)", text):
        sizes[m.group(1)] = int(m.group(2))
    return sizes


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_fp6_tiled_kernels_spill_no_more_than_pinned():
    sizes = {k: v for k, v in _scratch_sizes("fp6_gemm.hip").items() if "gemm_kernel" in k}
    assert len(sizes) == 7, sizes
    for name, scratch in sizes.items():
        # template arguments <BM, D, WN, DQ, FGQ, FMT, GBN, KW, DX> are mangled as ILi<BM>ELi<D>E...
        big = "ILi128ELi3ELi1ELi0ELb0ELi6ELi8E" in name
        assert scratch <= (8 if big else 0), (name, scratch)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_decode_kernels_do_not_spill():
    sizes = {k: v for k, v in _scratch_sizes("fp6_decode.hip").items() if "decode" in k}
    assert sizes and all(v == 0 for v in sizes.values()), sizes
