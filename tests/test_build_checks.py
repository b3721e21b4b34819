"""Host logic of the build: a spilling attention kernel is refused (its untracked LDS reads would be unsafe)."""
import pytest

from paper_2604_03260_amd import build

GOOD = """x.hip:1:1: remark: Function Name: _ZN5focus16attn_mfma_kernelILi128EEEvv [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     VGPRs: 244 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
x.hip:2:1: remark: Function Name: _ZN5focus15gather_k_kernelILi64EEEvv [-Rpass-analysis=kernel-resource-usage]
x.hip:2:1: remark:     VGPRs Spill: 3 [-Rpass-analysis=kernel-resource-usage]
"""


def test_accepts_a_build_without_spills_in_the_attention_kernel():
    assert build.check_no_spills(GOOD) == 1          # other kernels may spill: their loads are tracked


@pytest.mark.parametrize("bad", [
    GOOD.replace("VGPRs Spill: 0", "VGPRs Spill: 16"),
    GOOD.replace("ScratchSize [bytes/lane]: 0", "ScratchSize [bytes/lane]: 64"),
    GOOD.replace("attn_mfma_kernel", "some_other_kernel"),          # no report for the kernel at all
])
def test_refuses_spills_and_missing_reports(bad):
    with pytest.raises(RuntimeError):
        build.check_no_spills(bad)


def test_the_library_build_never_ablates_the_attention_loop():
    """FOCUS_ABLATE (timing-only builds of the loop ablation) defaults to 0 in the source and is set by
    build_ablation alone, which writes to another file than the library."""
    import os
    import re
    src = open(os.path.join(build.CSRC, "focus_attn_mfma.hip")).read()
    assert re.search(r"#ifndef FOCUS_ABLATE\s*\n#define FOCUS_ABLATE 0\s*\n#endif", src)
    assert not any("FOCUS_ABLATE" in f for f in build.FLAGS)
    import inspect
    assert "FOCUS_ABLATE" not in inspect.getsource(build.build_library)
    assert "libfocus_ablate_%d.so" in inspect.getsource(build.build_ablation)
