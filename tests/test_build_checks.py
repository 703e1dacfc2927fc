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


# ---- stage loads per K loop ------------------------------------------------------------------
def _k_loop(mode: int, n_loads: int, extra: str = "") -> str:
    loads = "".join("\tglobal_load_lds_dwordx4 v[2:3], off\n\tv_mfma_f32_32x32x16_bf16 v[20:35], v[10:13], v[10:13], v[20:35]\n"
                    for _ in range(n_loads))
    return (f"_ZN5jitdb12_GLOBAL__N_112level_kernelItLi{mode}ELb0ELb0EEEvNS_9LevelArgsE:\n"
            "\ts_load_dwordx2 s[0:1], s[4:5], 0x0\n"
            ".LBB0_1:\n" + loads + extra +
            "\ts_waitcnt vmcnt(6) lgkmcnt(0)\n\ts_barrier\n"
            "\ts_cbranch_scc1 .LBB0_1\n"
            "\tglobal_store_dwordx4 v[0:1], v[20:23], off\n"
            "\ts_endpgm\n")


def test_stage_load_count_per_k_loop():
    assert B.check_stage_loads(_k_loop(1, 6)) == 1          # internal / projection / plain GEMM: 6 per stage
    assert B.check_stage_loads(_k_loop(0, 5)) == 1          # leaf: 5
    with pytest.raises(RuntimeError, match="assume 6 per stage"):
        B.check_stage_loads(_k_loop(1, 5))
    with pytest.raises(RuntimeError, match="assume 5 per stage"):
        B.check_stage_loads(_k_loop(0, 6))


def test_foreign_vector_memory_instruction_in_a_k_loop_is_refused():
    with pytest.raises(RuntimeError, match="besides the stage loads"):
        B.check_stage_loads(_k_loop(1, 6, extra="\tglobal_load_dwordx4 v[40:43], v[2:3], off\n"))
    with pytest.raises(RuntimeError, match="besides the stage loads"):
        B.check_stage_loads(_k_loop(1, 6, extra="\tglobal_store_dword v[2:3], v40, off\n"))
    # the same instructions outside the loop are none of its business
    assert B.check_stage_loads(_k_loop(1, 6)) == 1
