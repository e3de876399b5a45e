"""The static checks the build runs over the compiled kernels (paper_2505_16162_amd/isa_check.py), tried on
small hand-written assembly texts: a correct rolling stream passes, planted mistakes are found."""
from paper_2505_16162_amd import isa_check as C

HEAD = "_ZN2ks11gemv_kernelEv:\n"
TAIL = "\ts_endpgm\n.Lfunc_end0:\n"


def asm_load(dst, addr, nt=True):
    return f"\t;;#ASMSTART\n\tglobal_load_dwordx4 {dst}, {addr}, off{' nt' if nt else ''}\n\t;;#ASMEND\n"


def asm_wait(n):
    return f"\t;;#ASMSTART\n\ts_waitcnt vmcnt({n})\n\t;;#ASMEND\n"


def body_of(text):
    (name, body), = C.kernel_bodies(HEAD + text + TAIL, "gemv_kernel")
    assert name.startswith("_ZN2ks11gemv_kernel")
    return body


def rolling_loop(use_before_wait=False, copy_in_flight=False, short_wait=False):
    """Two registers in flight; each is waited for (leaving the one younger load in flight), used and refilled."""
    t = asm_load("v[2:5]", "v[10:11]") + asm_load("v[6:9]", "v[12:13]")
    t += ".LBB0_1:\n"
    if use_before_wait:
        t += "\tv_add_f32_e32 v20, v20, v2\n"
    if copy_in_flight:
        t += "\tv_mov_b32_e32 v30, v6\n"
    t += asm_wait(1)
    t += "\tv_add_f32_e32 v20, v20, v2\n" + asm_load("v[2:5]", "v[10:11]")
    t += asm_wait(2 if short_wait else 1)
    t += "\tv_add_f32_e32 v20, v20, v6\n" + asm_load("v[6:9]", "v[12:13]")
    t += "\ts_cbranch_scc1 .LBB0_1\n"
    t += asm_wait(0) + "\tv_add_f32_e32 v20, v2, v6\n"
    return t


def test_clean_stream_has_no_flags():
    body = body_of(rolling_loop())
    assert C.inflight_flags(body) == []
    assert C.weight_register_copies(body) == []


def test_use_before_the_wait_is_flagged():
    flags = C.inflight_flags(body_of(rolling_loop(use_before_wait=True)))
    assert flags and any("v_add_f32_e32 v20, v20, v2" in t for _, t, _, _ in flags)


def test_wait_that_keeps_too_many_loads_is_flagged():
    # vmcnt(2) with only one younger load in flight does not retire v[6:9]
    flags = C.inflight_flags(body_of(rolling_loop(short_wait=True)))
    assert any(r in (6, 7, 8, 9) for _, _, r, _ in flags)


def test_copy_of_a_register_in_flight_is_flagged_by_both_checks():
    body = body_of(rolling_loop(copy_in_flight=True))
    assert any("v_mov_b32_e32 v30, v6" in t for _, t, _, _ in C.inflight_flags(body))
    assert [t for _, t in C.weight_register_copies(body)] == ["v_mov_b32_e32 v30, v6"]


def test_writing_a_weight_register_after_the_drain_is_not_a_copy():
    t = asm_load("v[2:5]", "v[10:11]") + asm_wait(0) + "\tv_mov_b32_e32 v2, v40\n" + asm_wait(0)
    assert C.weight_register_copies(body_of(t)) == []
    assert C.inflight_flags(body_of(t)) == []


def test_compiler_waits_do_not_retire_hand_placed_loads():
    t = asm_load("v[2:5]", "v[10:11]") + "\ts_waitcnt vmcnt(0)\n\tv_add_f32_e32 v20, v20, v2\n"
    assert C.inflight_flags(body_of(t))


def test_paths_are_merged_with_the_least_count():
    # one path issues a younger load, the other does not: vmcnt(1) is only safe on the first
    t = asm_load("v[2:5]", "v[10:11]") + "\ts_cbranch_scc1 .LBB0_2\n" + asm_load("v[6:9]", "v[12:13]")
    t += ".LBB0_2:\n" + asm_wait(1) + "\tv_add_f32_e32 v20, v20, v2\n" + asm_wait(0)
    assert any(r == 2 for _, _, r, _ in C.inflight_flags(body_of(t)))
