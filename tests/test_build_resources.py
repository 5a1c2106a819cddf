"""What the compiler reported about the kernels when the library was built: no kernel may keep
registers in scratch memory (a spill turns every use into memory traffic inside the hot loops;
it has cost single instantiations up to 28 % without failing any parity test)."""
import os

import pytest

import __graft_entry__ as entry

REPORT = os.path.join(entry.PKG, "_build", "kernel_resources.txt")

SAMPLE = """\
a.hip:5:1: remark: Function Name: _Z5alphav [-Rpass-analysis=kernel-resource-usage]
    5 | __global__ void alpha() {
      | ^
a.hip:5:1: remark:     TotalSGPRs: 16 [-Rpass-analysis=kernel-resource-usage]
a.hip:5:1: remark:     VGPRs: 74 [-Rpass-analysis=kernel-resource-usage]
a.hip:5:1: remark:     AGPRs: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:5:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:5:1: remark:     Dynamic Stack: False [-Rpass-analysis=kernel-resource-usage]
a.hip:5:1: remark:     Occupancy [waves/SIMD]: 6 [-Rpass-analysis=kernel-resource-usage]
a.hip:5:1: remark:     SGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark: Function Name: _Z4betav [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark:     VGPRs: 128 [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark:     ScratchSize [bytes/lane]: 68 [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark:     Occupancy [waves/SIMD]: 4 [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: warning: something else
"""


def test_resource_remarks_are_parsed():
    assert entry.kernel_resources(SAMPLE) == {"_Z5alphav": (74, 0, 6), "_Z4betav": (128, 68, 4)}
    assert entry.kernel_resources("") == {}


def test_no_kernel_spills_registers():
    if not os.path.exists(REPORT):
        pytest.skip("the library in the tree was not built by build() of this version: no resource report")
    rows = [l.split() for l in open(REPORT) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 100, "the report lists fewer kernels than the library has"
    spilled = [(r[0], int(r[2])) for r in rows if int(r[2]) != 0]
    assert not spilled, spilled
