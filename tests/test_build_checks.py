"""The build step's register-budget check (host logic only: the remark text is made up here)."""
from paper_2201_12023_amd import build as B

BATCH = "_ZN4alpa22recurrence_fast_kernelILi4ELi1ELi1ELb0ELb0ELb0ELb0EEEvNS_7ProblemEPKi"
PLAN = "_ZN4alpa22recurrence_fast_kernelILi4ELi4ELi1ELb1ELb0ELb0ELb0EEEvNS_7ProblemEPKi"
OTHER = "_ZN4alpa15epilogue_kernelENS_7ProblemEPKi"


def remarks(name, vgprs, scratch, occupancy):
    tag = " [-Rpass-analysis=kernel-resource-usage]"
    return "\n".join([
        f"remark: a.hpp:1:1: Function Name: {name}{tag}",
        f"remark: a.hpp:1:1:     TotalSGPRs: 94{tag}",
        f"remark: a.hpp:1:1:     VGPRs: {vgprs}{tag}",
        f"remark: a.hpp:1:1:     AGPRs: 0{tag}",
        f"remark: a.hpp:1:1:     ScratchSize [bytes/lane]: {scratch}{tag}",
        f"remark: a.hpp:1:1:     Occupancy [waves/SIMD]: {occupancy}{tag}",
    ]) + "\n"


def test_remarks_are_parsed_per_kernel():
    k = B.parse_resource_remarks(remarks(BATCH, 64, 0, 8) + remarks(OTHER, 30, 16, 8))
    assert k[BATCH] == {"vgprs": 64, "scratch": 0, "occupancy": 8}
    assert k[OTHER] == {"vgprs": 30, "scratch": 16, "occupancy": 8}


def test_batch_instance_must_keep_eight_waves_and_no_scratch():
    ok = B.parse_resource_remarks(remarks(BATCH, 64, 0, 8) + remarks(PLAN, 72, 0, 7) + remarks(OTHER, 30, 16, 8))
    assert B.check_resources(ok) == []
    assert len(B.check_resources(B.parse_resource_remarks(remarks(BATCH, 68, 0, 7)))) == 1
    assert len(B.check_resources(B.parse_resource_remarks(remarks(BATCH, 64, 24, 8)))) == 1
    # other instances of the recurrence kernel: any occupancy, but nothing in scratch
    assert len(B.check_resources(B.parse_resource_remarks(remarks(PLAN, 72, 12, 7)))) == 1
