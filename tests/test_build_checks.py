"""The build step's register-budget check (host logic only: the remark text is made up here)."""
from paper_2201_12023_amd import build as B

BATCH = "_ZN4alpa22recurrence_fast_kernelILi4ELi1ELi1ELb0ELb0ELb0ELb0EEEvNS_7ProblemEPKi"
PLAN = "_ZN4alpa22recurrence_fast_kernelILi4ELi4ELi1ELb1ELb0ELb0ELb0EEEvNS_7ProblemEPKi"
OTHER = "_ZN4alpa15epilogue_kernelENS_7ProblemEPKi"


def remarks(name, vgprs, scratch, occupancy, agprs=0):
    tag = " [-Rpass-analysis=kernel-resource-usage]"
    return "\n".join([
        f"remark: a.hpp:1:1: Function Name: {name}{tag}",
        f"remark: a.hpp:1:1:     TotalSGPRs: 94{tag}",
        f"remark: a.hpp:1:1:     VGPRs: {vgprs}{tag}",
        f"remark: a.hpp:1:1:     AGPRs: {agprs}{tag}",
        f"remark: a.hpp:1:1:     ScratchSize [bytes/lane]: {scratch}{tag}",
        f"remark: a.hpp:1:1:     Occupancy [waves/SIMD]: {occupancy}{tag}",
    ]) + "\n"


def test_remarks_are_parsed_per_kernel():
    k = B.parse_resource_remarks(remarks(BATCH, 64, 0, 8) + remarks(OTHER, 30, 16, 8))
    assert k[BATCH] == {"vgprs": 64, "agprs": 0, "scratch": 0, "occupancy": 8}
    assert k[OTHER] == {"vgprs": 30, "agprs": 0, "scratch": 16, "occupancy": 8}


def test_batch_instance_must_keep_eight_waves_and_no_scratch():
    ok = B.parse_resource_remarks(remarks(BATCH, 64, 0, 8) + remarks(PLAN, 72, 0, 7) + remarks(OTHER, 30, 16, 8))
    assert B.check_resources(ok) == []
    assert len(B.check_resources(B.parse_resource_remarks(remarks(BATCH, 68, 0, 7)))) == 1
    assert len(B.check_resources(B.parse_resource_remarks(remarks(BATCH, 64, 24, 8)))) == 1
    # other instances of the recurrence kernel: any occupancy, but nothing spilled, neither to
    # scratch memory nor to accumulation registers
    assert len(B.check_resources(B.parse_resource_remarks(remarks(PLAN, 72, 12, 7)))) == 1
    assert len(B.check_resources(B.parse_resource_remarks(remarks(PLAN, 72, 0, 7, agprs=4)))) == 1


ASM_HEAD = "\t.text\n_ZN4alpa22recurrence_fast_kernelILi4ELi1ELi1ELb0ELb0ELb0ELb0EEEvNS_7ProblemE: ; @x\n"


def kernel_asm(middle):
    return ASM_HEAD + "\n".join([
        "\tv_mov_b32_e32 v33, v18",            # another value in the register, before its time
        "\tv_mov_b32_e32 v33, 0",
        "\t;;#ASMSTART", "\tglobal_load_dword v33, v[14:15], off", "\t;;#ASMEND",
        *middle,
        "\t;;#ASMSTART", "\tglobal_load_dword v33, v[16:17], off", "\t;;#ASMEND",
        "\tv_min3_i32 v27, v27, v45, v46",
        "\t;;#ASMSTART", "\ts_waitcnt vmcnt(0)", "\t;;#ASMEND",
        "\tv_mov_b32_e32 v33, s30",            # free again behind the wait
        "\ts_endpgm", ""])


def test_warm_up_register_must_keep_its_place():
    assert B.check_warm_register(kernel_asm(["\tv_mov_b32_e32 v33, 0", "\tv_add_u32_e32 v45, s4, v12"])) == []
    # another value written into it between the loads and the wait
    assert len(B.check_warm_register(kernel_asm(["\tv_add_u32_e32 v33, s4, v12"]))) == 1
    assert len(B.check_warm_register(kernel_asm(["\tds_read2st64_b32 v[32:33], v44 offset0:2 offset1:3"]))) == 1
    # reading it is harmless; a compare writes no vector register
    assert B.check_warm_register(kernel_asm(["\tv_cmp_le_i32_e32 vcc, s1, v33"])) == []
    # loads into two registers, or no wait behind them
    two = kernel_asm([]).replace("global_load_dword v33, v[16:17]", "global_load_dword v40, v[16:17]")
    assert len(B.check_warm_register(two)) == 1
    assert len(B.check_warm_register(kernel_asm([]).replace("s_waitcnt vmcnt(0)", "s_nop 0"))) == 1
    # kernels without warm-up loads are not looked at
    assert B.check_warm_register(ASM_HEAD + "\tv_mov_b32_e32 v1, 0\n\ts_endpgm\n") == []
