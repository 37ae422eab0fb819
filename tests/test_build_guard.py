"""Host logic of the build: the parser that refuses kernels which use scratch memory."""
import pytest

from paper_2309_14717_amd import build as b

REMARK = """x.hip:1:1: remark: Function Name: {name} [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     VGPRs: 100 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     ScratchSize [bytes/lane]: {scratch} [-Rpass-analysis=kernel-resource-usage]
"""


def test_clean_kernels_pass():
    text = REMARK.format(name="_ZN6qalora14gemm_dq_kernelILi4EEEv", scratch=0)
    b._check_no_scratch("gemm_dq.hip", text)


def test_spilling_kernel_is_refused():
    text = REMARK.format(name="_ZN6qalora14gemm_dq_kernelILi4EEEv", scratch=48)
    with pytest.raises(RuntimeError, match="scratch"):
        b._check_no_scratch("gemm_dq.hip", text)


def test_only_listed_kernels_are_checked():
    # another kernel of the same file may spill (it is not hand-scheduled)
    text = REMARK.format(name="_ZN6qalora12merge_kernelILi8EEEv", scratch=16)
    b._check_no_scratch("adapter.hip", text)
    text = REMARK.format(name="_ZN6qalora12front_kernelENS_9FrontArgsE", scratch=16)
    with pytest.raises(RuntimeError):
        b._check_no_scratch("adapter.hip", text)
