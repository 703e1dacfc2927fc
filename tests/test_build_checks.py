"""The build's static checks on generated code (host logic, no GPU)."""
import pytest

from paper_1904_07421_amd import build as B

GOOD = """
_ZN5jitdb12level_kernelEv:
\ts_load_dwordx2 s[0:1], s[4:5], 0x0
\ts_waitcnt lgkmcnt(0)
.LBB0_1:
\tds_read_b128 v[10:13], v1
\tds_read_b128 v[14:17], v2 offset:2048
\tv_add_u32_e32 v3, 1, v3
\ts_waitcnt lgkmcnt(1)
\tv_mfma_f32_32x32x16_bf16 v[20:35], v[10:13], v[10:13], v[20:35]
\ts_waitcnt lgkmcnt(0)
\tv_mfma_f32_32x32x16_bf16 v[20:35], v[14:17], v[14:17], v[20:35]
\ts_cbranch_scc1 .LBB0_1
\ts_endpgm
"""


def test_clean_code_passes_and_reads_are_counted():
    assert B.check_lds_read_waits(GOOD) == 2


def test_copy_of_a_register_in_flight_is_refused():
    bad = GOOD.replace("\tv_add_u32_e32 v3, 1, v3\n", "\tv_mov_b32_e32 v40, v15\n")
    with pytest.raises(RuntimeError, match="in flight"):
        B.check_lds_read_waits(bad)


def test_wait_that_covers_only_the_older_read_is_not_enough():
    bad = GOOD.replace("\ts_waitcnt lgkmcnt(0)\n\tv_mfma_f32_32x32x16_bf16 v[20:35], v[14:17]",
                       "\tv_mfma_f32_32x32x16_bf16 v[20:35], v[14:17]")
    with pytest.raises(RuntimeError, match="in flight"):
        B.check_lds_read_waits(bad)


def test_state_follows_the_back_edge():
    # the read at the loop's end is still in flight when the loop head uses its register
    bad = GOOD.replace("\ts_cbranch_scc1 .LBB0_1\n", "\tds_read_b128 v[3:6], v2\n\ts_cbranch_scc1 .LBB0_1\n")
    with pytest.raises(RuntimeError, match="in flight"):
        B.check_lds_read_waits(bad)


def test_other_kernels_are_not_examined():
    other = GOOD.replace("level_kernel", "stack_kernel").replace("\ts_waitcnt lgkmcnt(1)\n", "")
    assert B.check_lds_read_waits(other) == 0


def test_spilling_kernel_is_refused():
    lines = ["remark: x.hip:1:1: Function Name: k1 [-Rpass-analysis=kernel-resource-usage]",
             "remark: x.hip:1:1:     ScratchSize [bytes/lane]: 16 [-Rpass-analysis=kernel-resource-usage]"]
    with pytest.raises(RuntimeError, match="scratch"):
        B._check_no_scratch(lines)
    B._check_no_scratch([l.replace(": 16 ", ": 0 ") for l in lines])
