"""The build's check of hand-issued loads in the generated code, on small pieces of assembly text."""
import importlib.util
import os

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
_spec = importlib.util.spec_from_file_location(
    "verify_hand_loads", os.path.join(HERE, "..", "paper_2506_04642_amd", "verify_hand_loads.py"))
v = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(v)

HEAD = "_ZN6tadakv24decode_split_mfma_kernelILi8EEEvNS_10DecodeArgsE:\n"
TAIL = "\ts_endpgm\n.Lfunc_end0:\n"


def kernel(body):
    return HEAD + body + TAIL


GOOD = kernel("""
	;;#ASMSTART
	global_load_dwordx4 a[0:3], v[28:29], off ; by hand
	;;#ASMEND
	v_add_u32_e32 v4, v5, v6
	;;#ASMSTART
	s_waitcnt vmcnt(18)
	;;#ASMEND
	;;#ASMSTART
	; by hand a[0:3]
	;;#ASMEND
	v_accvgpr_read_b32 v10, a0
	;;#ASMSTART
	ds_read_b128 v[40:43], v7 offset:64
	;;#ASMEND
	v_add_u32_e32 v4, v5, v6
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
	v_mov_b32_e32 v9, v40
""")


def test_untouched_destinations_pass():
    problems, kernels, n, nl = v.check_text(GOOD)
    assert problems == [] and kernels == 1 and n == 1 and nl == 1


def test_a_copy_before_the_hand_over_is_found():
    # the destination is copied into the accumulation file before the data can be there
    bad = kernel("""
	;;#ASMSTART
	global_load_dwordx4 v[8:11], v[28:29], off ; by hand
	;;#ASMEND
	v_accvgpr_write_b32 a63, v11
	;;#ASMSTART
	s_waitcnt vmcnt(0)
	;;#ASMEND
	;;#ASMSTART
	; by hand v[8:11]
	;;#ASMEND
""")
    problems, _, _, _ = v.check_text(bad)
    assert len(problems) == 1 and "v_accvgpr_write_b32 a63, v11" in problems[0]


def test_a_hand_over_under_another_name_is_found():
    bad = kernel("""
	;;#ASMSTART
	global_load_dwordx4 a[0:3], v[28:29], off ; by hand
	;;#ASMEND
	;;#ASMSTART
	; by hand a[4:7]
	;;#ASMEND
""")
    problems, _, _, _ = v.check_text(bad)
    assert any("which no request names" in p for p in problems)
    assert any("never handed over" in p for p in problems)


def test_scratch_traffic_and_early_use_of_an_lds_read_are_found():
    bad = kernel("""
	;;#ASMSTART
	global_load_dwordx4 a[0:3], v[28:29], off ; by hand
	;;#ASMEND
	scratch_store_dword off, v3, s32
	;;#ASMSTART
	; by hand a[0:3]
	;;#ASMEND
	;;#ASMSTART
	ds_read_b128 v[40:43], v7
	;;#ASMEND
	v_mov_b32_e32 v9, v41
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
""")
    problems, _, _, _ = v.check_text(bad)
    assert any("scratch access" in p for p in problems)
    assert any("LDS read" in p for p in problems)


def test_a_file_without_hand_loads_is_refused(tmp_path):
    f = tmp_path / "empty.s"
    f.write_text(kernel("\tv_mov_b32_e32 v0, v1\n"))
    with pytest.raises(RuntimeError):
        v.verify(str(f))
    g = tmp_path / "good.s"
    g.write_text(GOOD)
    assert v.verify(str(g)) == (1, 1, 1)
