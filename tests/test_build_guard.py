"""The build refuses a library whose hand-counted waits for memory no longer match the generated code.

The level-major propagation kernels wait with ``s_waitcnt vmcnt(N)`` for "everything but the last N memory
instructions"; that is only right while the compiler issues exactly the loads and stores the source shows between two
such waits.  ``build.check_counted_waits`` reads the device assembly; here it is run on the real assembly and on copies
of it with one mistake planted in each.
"""
import os
import re

import pytest

from paper_1803_03288_amd import build as b


@pytest.fixture(scope="module")
def asm():
    return b.device_assembly(os.path.join(b.CSRC, "k1_propagate.hip"))


def function_span(asm, key):
    start = next(m.start() for m in re.finditer(r"^_Z\S*:", asm, re.M) if key in m.group(0))
    return start, asm.index(".Lfunc_end", start)


def hand_waits(text, n):
    return [m.start() for m in re.finditer(r";;#ASMSTART\s+s_waitcnt vmcnt\(%d\)" % n, text)]


def test_generated_code_matches_the_counts(asm):
    assert b.check_counted_waits(asm) == []


@pytest.mark.parametrize("key,n", [("16propagate_levelsILi1", 21), ("24propagate_levels_q_batchILi4", 14)])
def test_a_missing_load_between_two_waits_is_found(asm, key, n):
    lo, hi = function_span(asm, key)
    body = asm[lo:hi]
    w = hand_waits(body, n)
    piece = body[w[3]:w[4]]
    assert "global_load_dwordx4" in piece
    broken = body[:w[3]] + piece.replace("global_load_dwordx4", "; global_load_dwordx4", 1) + body[w[4]:]
    bad = b.check_counted_waits(asm[:lo] + broken + asm[hi:])
    assert any(key in x and "between two waits" in x for x in bad)


def test_a_spill_is_found(asm):
    lo, hi = function_span(asm, "22propagate_levels_batchILi4")
    body = asm[lo:hi]
    w = hand_waits(body, 21)
    broken = body[:w[2]] + "\tscratch_load_dword v2, off, off offset:8\n" + body[w[2]:]
    bad = b.check_counted_waits(asm[:lo] + broken + asm[hi:])
    assert any("spills" in x for x in bad)


def test_another_count_is_found(asm):
    lo, hi = function_span(asm, "16propagate_levelsILi2")
    body = asm[lo:hi].replace("s_waitcnt vmcnt(21)", "s_waitcnt vmcnt(24)", 1)
    bad = b.check_counted_waits(asm[:lo] + body + asm[hi:])
    assert any("is not vmcnt(21)" in x for x in bad)


def test_a_store_after_the_request_is_found(asm):
    lo, hi = function_span(asm, "15propagate_nodesILi1")
    body = asm[lo:hi]
    w = hand_waits(body, 8)
    assert len(w) >= 2
    broken = body[:w[1]] + "\tglobal_store_dwordx2 v[4:5], v[2:3], off\n" + body[w[1]:]
    bad = b.check_counted_waits(asm[:lo] + broken + asm[hi:])
    assert any("15propagate_nodesILi1" in x for x in bad)


def test_a_kernel_that_is_gone_is_found(asm):
    bad = b.check_counted_waits(asm.replace("propagate_levels_q_batch", "propagate_levels_x_batch"))
    assert any("24propagate_levels_q_batchILi" in x for x in bad)
