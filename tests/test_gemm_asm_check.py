"""The build's static checker for the batched kernel's hand-counted loads: it must accept a
correctly waited load and flag the hazards it exists for (planted here, in text, on the CPU)."""
import os

from paper_2407_21082_amd import check_gemm_asm as C

NAME = "_ZN2eh12_GLOBAL__N_117gemm_stats_kernelINS_6DtBf16ELi1ELb0EEEvPKDv4_jS5_iiiPKiiiPNS_5StatsE"


def kernel(body: str) -> str:
    return f"{NAME}:\n{body}\n.Lfunc_end0:\n"


STEP_OK = """
\ts_waitcnt vmcnt(3) lgkmcnt(0) ; step-sync
\ts_barrier
.LBB0_1:
\tglobal_load_lds_dwordx4 v[2:3], off
\tglobal_load_lds_dwordx4 v[4:5], off
\tv_mfma_f32_16x16x32_bf16 a[0:3], v[20:23], v[8:11], a[0:3]
\t;;#ASMSTART
\tglobal_load_dwordx4 v[8:11], v[6:7], off
\t;;#ASMEND
\ts_waitcnt vmcnt(3) lgkmcnt(0) ; step-sync
\ts_barrier
\tglobal_load_lds_dwordx4 v[2:3], off
\tglobal_load_lds_dwordx4 v[4:5], off
\tv_mfma_f32_16x16x32_bf16 a[0:3], v[20:23], v[12:15], a[0:3]
\t;;#ASMSTART
\tglobal_load_dwordx4 v[12:15], v[6:7], off
\t;;#ASMEND
\ts_waitcnt vmcnt(3) lgkmcnt(0) ; step-sync
\ts_barrier
\ts_cbranch_scc1 .LBB0_1
\ts_waitcnt vmcnt(0)
\ts_endpgm
"""


def test_accepts_counted_waits():
    findings, nk, nl = C.check_asm(kernel(STEP_OK))
    assert nk == 1 and nl == 2
    assert findings == []


def test_flags_destination_reused_while_in_flight():
    # the address of a later DMA load is computed into the in-flight destination
    bad = STEP_OK.replace("\ts_cbranch_scc1 .LBB0_1\n",
                          "\ts_cbranch_scc1 .LBB0_1\n\tv_lshl_add_u64 v[12:13], v[30:31], 0, s[0:1]\n")
    findings, _, _ = C.check_asm(kernel(bad))
    assert any("v_lshl_add_u64 v[12:13]" in f for f in findings)


def test_flags_use_before_the_wait():
    # an MFMA hoisted above the wait that covers its operand
    bad = STEP_OK.replace("\tglobal_load_dwordx4 v[12:15], v[6:7], off\n\t;;#ASMEND\n",
                          "\tglobal_load_dwordx4 v[12:15], v[6:7], off\n\t;;#ASMEND\n"
                          "\tv_mfma_f32_16x16x32_bf16 a[0:3], v[20:23], v[12:15], a[0:3]\n")
    findings, _, _ = C.check_asm(kernel(bad))
    assert any("touches its destination" in f for f in findings)


def test_flags_load_in_flight_at_end_and_wrong_step_count():
    bad = STEP_OK.replace("\ts_waitcnt vmcnt(0)\n\ts_endpgm", "\ts_endpgm")
    findings, _, _ = C.check_asm(kernel(bad))
    assert any("in flight at s_endpgm" in f for f in findings)
    extra = STEP_OK.replace("\tglobal_load_dwordx4 v[12:15], v[6:7], off\n\t;;#ASMEND\n",
                            "\tglobal_load_dwordx4 v[12:15], v[6:7], off\n\t;;#ASMEND\n\tglobal_load_dword v40, v[6:7], off\n")
    findings, _, _ = C.check_asm(kernel(extra))
    assert any("other vector memory" in f for f in findings)


def test_a_store_does_not_count_as_a_younger_load():
    bad = STEP_OK.replace("\tglobal_load_lds_dwordx4 v[4:5], off\n\tv_mfma_f32_16x16x32_bf16 a[0:3], v[20:23], v[12:15]",
                          "\tglobal_store_dword v[4:5], v40, off\n\tv_mfma_f32_16x16x32_bf16 a[0:3], v[20:23], v[12:15]")
    findings, _, _ = C.check_asm(kernel(bad))
    assert findings


def test_only_inline_asm_loads_are_hand_counted():
    """A 16-byte load the compiler emitted itself is tracked by the compiler's own wait counts: it may
    overwrite a destination whose value is dead while the first load is still on its way (loads return
    in order).  The same two instructions inside inline-asm markers are a hazard."""
    tail_ok = ("\ts_waitcnt vmcnt(0)\n\tglobal_load_dwordx4 v[50:53], v[6:7], off\n\tglobal_load_dwordx2 v[50:51], v[6:7], off\n"
               "\ts_waitcnt vmcnt(0)\n\ts_endpgm")
    ok = STEP_OK.replace("\ts_waitcnt vmcnt(0)\n\ts_endpgm", tail_ok)
    findings, _, nl = C.check_asm(kernel(ok))
    assert findings == [] and nl == 2
    tail_bad = ("\ts_waitcnt vmcnt(0)\n\t;;#ASMSTART\n\tglobal_load_dwordx4 v[50:53], v[6:7], off\n\t;;#ASMEND\n"
                "\tglobal_load_dwordx2 v[50:51], v[6:7], off\n\ts_waitcnt vmcnt(0)\n\ts_endpgm")
    findings, _, nl = C.check_asm(kernel(STEP_OK.replace("\ts_waitcnt vmcnt(0)\n\ts_endpgm", tail_bad)))
    assert nl == 3 and any("touches its destination" in f for f in findings)


def test_built_library_was_checked():
    """The assembly the in-tree library was built from, if a build left it, is clean."""
    build_dir = os.path.join(os.path.dirname(C.__file__), "_build")
    paths = [os.path.join(build_dir, n) for n in ("eh_gemm.s", "eh_gemm32.s")]
    if not all(os.path.exists(p) for p in paths):
        import pytest
        pytest.skip("no build directory (library built elsewhere)")
    for path in paths:
        findings, nk, nl = C.check_asm(open(path).read())
        assert nk >= 4 and nl > 0 and findings == [], path
