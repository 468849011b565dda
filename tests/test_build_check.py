"""The build's check of the generated assembly of the tile kernels (paper_2512_15306_amd/build.py): the MFMAs are
written out as inline assembly, so nothing but MFMAs may touch accumulator registers between the first MFMA and the
wait states behind the K loop.  Here the check itself is tested, on hand-written assembly text."""
import pytest

from paper_2512_15306_amd import build

NAME = "_ZN4llmq16gemm_tile_kernelILi0ELi0ELi4ELi4ELb0ENS_10GemmTuningELb0ELb0ELi0EEEvPKhS3_Pt"


def kernel(body: str, name: str = NAME) -> str:
    return "\t.text\n%s:                                ; @%s\n; %%bb.0:\n%s\n.Lfunc_end0:\n\t.size\t%s, .Lfunc_end0-%s\n" % (
        name, name, body, name, name)


GOOD = """\tv_mov_b32_e32 v5, 0
\tv_accvgpr_write_b32 a0, v5
\tv_accvgpr_write_b32 a1, v5
.LBB0_3:                                ; =>This Inner Loop Header: Depth=1
\tds_read_b128 v[10:13], v1
\ts_waitcnt lgkmcnt(0)
\tv_mfma_f32_16x16x128_f8f6f4 a[0:3], v[20:27], v[10:17], a[0:3]
\tbuffer_load_dwordx4 v2, s[8:11], s0 offen lds
\tv_mfma_f32_16x16x128_f8f6f4 a[4:7], v[20:27], v[10:17], a[4:7] blgp:1
\ts_cbranch_scc1 .LBB0_3
.LBB0_4:
\tv_accvgpr_write_b32 a8, v5
\tv_mfma_f32_16x16x128_f8f6f4 a[8:11], v[20:27], v[10:17], a[8:11]
\ts_nop 15
\ts_nop 15
\ts_waitcnt vmcnt(0)
\ts_barrier
\tv_accvgpr_read_b32 v30, a0
\tglobal_store_dwordx4 v[40:41], a[4:7], off
\ts_endpgm"""


def test_a_clean_kernel_passes():
    build.check_accumulator_reads("good.hip", kernel(GOOD))


@pytest.mark.parametrize("planted", [
    "\tv_accvgpr_read_b32 v30, a2",                                        # copy out of the accumulator file
    "\tscratch_store_dwordx4 off, a[4:7], off offset:16 ; 16-byte Folded Spill",
    "\tv_accvgpr_mov_b32 a9, a1",
    "\tscratch_load_dwordx4 a[0:3], off, off ; 16-byte Folded Reload",
    "\tv_accvgpr_write_b32 a3, 0",                                         # a constant the compiler re-creates
])
@pytest.mark.parametrize("where", ["in the loop", "behind the loop"])
def test_accumulator_access_inside_the_mfma_stretch_fails(planted, where):
    anchor = "\tbuffer_load_dwordx4 v2" if where == "in the loop" else "\ts_nop 15\n\ts_nop 15"
    bad = GOOD.replace(anchor, planted + "\n" + anchor, 1)
    assert bad != GOOD
    with pytest.raises(RuntimeError, match="accumulator registers touched"):
        build.check_accumulator_reads("bad.hip", kernel(bad))


def test_missing_wait_states_fail():
    with pytest.raises(RuntimeError, match="no wait states behind the last MFMA"):
        build.check_accumulator_reads("bad.hip", kernel(GOOD.replace("\ts_nop 15\n\ts_nop 15\n", "")))


def test_a_source_without_tile_kernels_fails():
    with pytest.raises(RuntimeError, match="no tile kernel found"):
        build.check_accumulator_reads("empty.hip", kernel(GOOD, name="_ZN4llmq19amax_partial_kernelEPKt"))


def test_kernels_without_mfma_are_skipped_but_others_still_count():
    adder = kernel("\tglobal_load_dwordx4 a[0:3], v[2:3], off\n\tv_accvgpr_read_b32 v1, a0\n\ts_endpgm", name=NAME.replace("Li0EEEv", "Li2EEEv"))
    build.check_accumulator_reads("mixed.hip", adder + kernel(GOOD))
    with pytest.raises(RuntimeError, match="no tile kernel found"):
        build.check_accumulator_reads("only_adder.hip", adder)
