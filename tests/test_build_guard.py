"""Host-side build logic (CPU only)."""
from paper_2412_18106_amd import build as B


def test_scratch_report_reads_the_compiler_remarks():
    text = ("a.hip:1:1: remark: Function Name: kernel_a [-Rpass-analysis=kernel-resource-usage]\n"
            "a.hip:1:1: remark:     VGPRs: 12 [-Rpass-analysis=kernel-resource-usage]\n"
            "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
            "a.hip:9:1: remark: Function Name: kernel_b [-Rpass-analysis=kernel-resource-usage]\n"
            "a.hip:9:1: remark:     ScratchSize [bytes/lane]: 148 [-Rpass-analysis=kernel-resource-usage]\n")
    assert B._scratch_report(text) == {"kernel_a": 0, "kernel_b": 148}
    assert B._scratch_report("") == {}
