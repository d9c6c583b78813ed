"""Host-side checks of the build: the spill check of the kernels with hand-issued matrix instructions."""
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
