"""The build writes the compiler's per-kernel resource report and refuses kernels that spill
registers to scratch memory (the kernels that count their own outstanding memory operations are
written for code without spills).  This checks the report of the library that is in the tree."""
import os

import pytest

from paper_2405_03133_amd import build


def test_no_kernel_uses_scratch_memory():
    if not os.path.exists(build.RESOURCES):
        pytest.skip("no build report in this tree (python -m paper_2405_03133_amd.build writes it)")
    rows = [ln.split() for ln in open(build.RESOURCES) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 100, len(rows)
    spilling = [(r[0], r[3]) for r in rows if int(r[3]) != 0]
    assert not spilling, spilling
    # every kernel family of the path is in the report
    names = " ".join(r[0] for r in rows)
    for family in ("gemm2_kernel", "fmg_kernel", "fmg8_kernel", "merge_kernel", "scatter_kernel", "route_mean_kernel",
                   "route_bwd_dx_kernel", "swiglu_bwd_kernel", "dw_reduce_kernel"):
        assert family in names, family


def test_report_parser_reads_the_compilers_remarks():
    text = "\n".join([
        "a.h:1:1: remark: Function Name: kern_a [-Rpass-analysis=kernel-resource-usage]",
        "a.h:1:1: remark:     VGPRs: 12 [-Rpass-analysis=kernel-resource-usage]",
        "a.h:1:1: remark:     AGPRs: 3 [-Rpass-analysis=kernel-resource-usage]",
        "a.h:1:1: remark:     ScratchSize [bytes/lane]: 16 [-Rpass-analysis=kernel-resource-usage]",
        "a.h:1:1: remark:     LDS Size [bytes/block]: 512 [-Rpass-analysis=kernel-resource-usage]",
    ])
    found = {}
    for ln in text.splitlines():
        m = build._REMARK.search(ln)
        assert m, ln
        found[m.group(1)] = m.group(2)
    assert found == {"Function Name": "kern_a", "VGPRs": "12", "AGPRs": "3", "ScratchSize [bytes/lane]": "16",
                     "LDS Size [bytes/block]": "512"}
