"""The build's check that no streaming kernel spills to scratch memory: the parser of the compiler's resource-usage remarks."""
from paper_2311_02103_amd.build import NO_SCRATCH, scratch_users, sources

REMARKS = """\
a.hip:17:1: remark: Function Name: _ZN5relax9gemv_q4_reg_kernelILi0EEEvv [-Rpass-analysis=kernel-resource-usage]
   17 | {
      | ^
a.hip:17:1: remark:     VGPRs: 79 [-Rpass-analysis=kernel-resource-usage]
a.hip:17:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:47:1: remark: Function Name: _ZN5relax9gemv_q4_reg_kernelILi1EEEvv [-Rpass-analysis=kernel-resource-usage]
a.hip:47:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]
a.hip:47:1: remark:     ScratchSize [bytes/lane]: 640 [-Rpass-analysis=kernel-resource-usage]
a.hip:60:1: remark: Function Name: _ZN5relax5otherEv [-Rpass-analysis=kernel-resource-usage]
a.hip:60:1: remark:     ScratchSize [bytes/lane]: 8 [-Rpass-analysis=kernel-resource-usage]
"""


def test_scratch_users_names_the_spilling_kernels_of_the_guarded_family_only():
    assert scratch_users(REMARKS, "gemv_q4_reg_kernel") == [("_ZN5relax9gemv_q4_reg_kernelILi1EEEvv", 640)]
    assert scratch_users(REMARKS, "other") == [("_ZN5relax5otherEv", 8)]
    assert scratch_users("", "gemv") == []


def test_every_guarded_source_exists():
    assert set(NO_SCRATCH) <= set(sources())
