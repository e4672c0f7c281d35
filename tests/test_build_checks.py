"""Host-side checks of the build script (no GPU)."""
from paper_2007_13055_amd import build


REMARKS = """\
a.hip:10:1: remark: Function Name: kernel_ok [-Rpass-analysis=kernel-resource-usage]
a.hip:10:1: remark:     VGPRs: 64 [-Rpass-analysis=kernel-resource-usage]
a.hip:10:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:10:1: remark:     SGPRs Spill: 12 [-Rpass-analysis=kernel-resource-usage]
a.hip:10:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:20:1: remark: Function Name: kernel_spills [-Rpass-analysis=kernel-resource-usage]
a.hip:20:1: remark:     ScratchSize [bytes/lane]: 188 [-Rpass-analysis=kernel-resource-usage]
a.hip:20:1: remark:     VGPRs Spill: 70 [-Rpass-analysis=kernel-resource-usage]
"""


def test_spill_detector_names_only_the_spilling_kernel():
    assert build._spilling_kernels(REMARKS) == ["kernel_spills"]
    assert build._spilling_kernels("") == []


def test_kernels_with_hand_placed_loads_are_checked():
    names = [s.rsplit("/", 1)[-1] for s in build.sources()]
    for f in build.NO_SPILL:
        assert f in names
