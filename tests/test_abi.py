"""CPU-only checks of the C-ABI library: it loads, exports every symbol that
include/tictac.h declares, and its host-side validation returns the documented
status codes (no kernel is launched here)."""

import ctypes
import os
import re

import numpy as np
import pytest

from paper_1803_03288_amd import binding, build as build_mod

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        build_mod.build()
    return binding.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tictac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tictac_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    names = declared_functions()
    assert "tictac_build_deps" in names and "tictac_simulate" in names and len(names) >= 10
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def _build(L, n, row_ptr, col_idx, recv_ids):
    rp = np.asarray(row_ptr, dtype=np.int32)
    ci = np.asarray(col_idx, dtype=np.int32)
    ri = np.asarray(recv_ids, dtype=np.int32)
    h = ctypes.c_void_p()
    rc = L.tictac_build_deps(ctypes.c_int32(n), rp.ctypes.data_as(ctypes.c_void_p),
                             ci.ctypes.data_as(ctypes.c_void_p), ctypes.c_int32(ri.size),
                             ri.ctypes.data_as(ctypes.c_void_p), None, ctypes.byref(h))
    return rc, h, L.tictac_last_error().decode()


def test_validation_status_codes(L):
    # cycle: op1 <- {recv0, op2}; op2 <- {op1}
    rc, h, msg = _build(L, 3, [0, 0, 2, 3], [0, 2, 1], [0])
    assert rc == -3 and "cycle" in msg and not h.value
    # row_ptr decreasing
    assert _build(L, 2, [0, 1, 0], [0], [])[0] == -2
    # row_ptr[0] != 0
    assert _build(L, 1, [1, 1], [0], [])[0] == -2
    # predecessor id out of range
    assert _build(L, 2, [0, 0, 1], [5], [0])[0] == -2
    # recv id out of range / duplicated / with predecessors
    assert _build(L, 2, [0, 0, 1], [0], [7])[0] == -2
    assert _build(L, 2, [0, 0, 1], [0], [0, 0])[0] == -5
    assert _build(L, 2, [0, 0, 1], [0], [1])[0] == -4
    # more recvs than ops, negative sizes
    assert _build(L, 1, [0, 0], [], [0, 0])[0] in (-2, -5)
    assert _build(L, -1, [0], [], [])[0] == -2
    # NULL pointers
    h = ctypes.c_void_p()
    assert L.tictac_build_deps(ctypes.c_int32(1), None, None, ctypes.c_int32(0), None, None, ctypes.byref(h)) == -1
    rp = np.zeros(2, dtype=np.int32)
    assert L.tictac_build_deps(ctypes.c_int32(1), rp.ctypes.data_as(ctypes.c_void_p), None, ctypes.c_int32(0),
                               None, None, None) == -1


def test_null_handle_is_rejected(L):
    assert L.tictac_dag_info(None, None, None, None, None, None) == -1
    assert L.tictac_tic_priority(None, None, None, None, None) == -1
    assert L.tictac_tac_priority(None, ctypes.c_int32(1), None, None, None, None, None, None, None) == -1
    assert L.tictac_simulate(None, ctypes.c_int32(1), None, ctypes.c_int32(0), None, None, None, None, None, None,
                             None, None) == -1
    assert L.tictac_dag_free(None) == 0
    # time oracle: no run, negative length, NULL buffers
    assert L.tictac_time_oracle_min(ctypes.c_int32(0), ctypes.c_int64(4), None, None, None) == -9
    assert L.tictac_time_oracle_min(ctypes.c_int32(5), ctypes.c_int64(-1), None, None, None) == -9
    assert L.tictac_time_oracle_min(ctypes.c_int32(5), ctypes.c_int64(4), None, None, None) == -1
    assert L.tictac_time_oracle_min(ctypes.c_int32(5), ctypes.c_int64(0), None, None, None) == 0
    # straggler effect: group size below 1, negative batch, NULL buffers with at least one group
    assert L.tictac_straggler_effect(ctypes.c_int32(8), ctypes.c_int32(0), None, None, None) == -9
    assert L.tictac_straggler_effect(ctypes.c_int32(-1), ctypes.c_int32(2), None, None, None) == -9
    assert L.tictac_straggler_effect(ctypes.c_int32(8), ctypes.c_int32(2), None, None, None) == -1
    assert L.tictac_straggler_effect(ctypes.c_int32(3), ctypes.c_int32(4), None, None, None) == 0     # no whole group
    # float32 timing arrays: no handle
    assert L.tictac_simulate_f32(None, ctypes.c_int32(1), None, ctypes.c_int32(0), None, None, None, None, None, None,
                                 None, None) == -1
    assert L.tictac_tac_simulate_f32(None, ctypes.c_int32(1), None, None, None, None, None, None, None, None, None,
                                     None, None, None) == -1
    # order search: no handle
    assert L.tictac_order_search(None, ctypes.c_int32(1), None, ctypes.c_int32(0), ctypes.c_int32(0), None, None, None,
                                 None, None, None, None, None) == -1
    assert binding.version().count(".") == 1
