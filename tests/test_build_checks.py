"""Host-side checks of the build: the spill check and the instruction-spacing check of the kernels with hand-issued
matrix instructions (both read compiler output as text; nothing runs on a GPU)."""
import pytest


def test_spill_check_refuses_scratch_and_vacuous_passes():
    from paper_2307_11339_amd import _build as B
    src = next(iter(B.NO_SPILL))
    kernel, piece = B.NO_SPILL[src]
    name = "_ZN3rnn12_GLOBAL__N_1%sINS_10TraitsBf16%sE" % (kernel, piece)
    ok = "remark: Function Name: %s [-Rpass-analysis]\nremark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis]\n" % name
    B._check_no_spill(src, ok)
    with pytest.raises(RuntimeError, match="spills"):
        B._check_no_spill(src, ok.replace("lane]: 0", "lane]: 24"))
    # remarks in which no kernel of that name appears must not pass for "nothing spilled"
    with pytest.raises(RuntimeError, match="checks nothing"):
        B._check_no_spill(src, ok.replace(kernel, "some_other_kernel"))
    with pytest.raises(RuntimeError, match="checks nothing"):
        B._check_no_spill(src, "")


def _hand(n, acc):
    return ";;#ASMSTART\n\tv_mfma_f32_16x16x32_bf16 a[%d:%d], a[200:203], v[8:11], a[%d:%d]\n;;#ASMEND\n" % (acc, acc + 3, acc, acc + 3) * n


def test_hand_issued_matrix_instruction_spacing_check():
    from paper_2307_11339_amd import _build as B
    head = "_Z6kernelv:\n\ts_load_dwordx2 s[0:1], s[4:5], 0x0\n"
    rotate = "".join(_hand(1, 4 * i) for i in range(B.HAND_MIN_APART)) * 3
    wait = ";;#ASMSTART\n\ts_nop 7\n\ts_nop 7\n\ts_nop 7\n;;#ASMEND\n"
    good = head + "\tv_accvgpr_write_b32 a0, 0\n\ts_nop 1\n" + rotate + wait + "\tds_write_b128 v1, a[0:3]\n\ts_endpgm\n"
    assert B._check_hand_issued("k.hip", good) == 3 * B.HAND_MIN_APART
    # the same accumulator again too soon
    with pytest.raises(RuntimeError, match="instructions apart"):
        B._check_hand_issued("k.hip", head + _hand(2, 0) + "\ts_endpgm\n")
    # the result read by something else before the instruction has delivered it
    with pytest.raises(RuntimeError, match="wait states after a hand-issued"):
        B._check_hand_issued("k.hip", head + rotate + "\ts_nop 3\n\tds_write_b128 v1, a[0:3]\n\ts_endpgm\n")
    with pytest.raises(RuntimeError, match="wait states after a hand-issued"):
        B._check_hand_issued("k.hip", head + rotate + "\tv_accvgpr_read_b32 v5, a%d\n\ts_endpgm\n" % (4 * B.HAND_MIN_APART - 1))
    # an accumulator set and used at once
    with pytest.raises(RuntimeError, match="after v_accvgpr_write"):
        B._check_hand_issued("k.hip", head + "\tv_accvgpr_write_b32 a2, 0\n" + _hand(1, 0) + "\ts_endpgm\n")
    # the compiler's own matrix instructions are its own business; code without any hand-issued one must not pass
    own = head + "\tv_mfma_f32_16x16x32_bf16 a[0:3], v[0:3], v[4:7], a[0:3]\n" * 2 + "\tds_write_b128 v1, a[0:3]\n\ts_endpgm\n"
    with pytest.raises(RuntimeError, match="checks nothing"):
        B._check_hand_issued("k.hip", own)
    # a load into the register in between makes it the load's value (the compiler waits for loads by itself)
    B._check_hand_issued("k.hip", head + rotate + "\tglobal_load_dwordx4 a[0:3], v[2:3], off\n\tds_write_b128 v1, a[0:3]\n\ts_endpgm\n")
