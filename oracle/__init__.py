"""CPU oracle of the TicTac scheduling math -- TEST INFRASTRUCTURE.

A numpy front-end to ``tictac_oracle.c`` (plain C, float64, single thread), the
slow and obviously-correct implementation that the GPU library is compared
with.  It shares no code with the GPU path and must only be used by the tests,
the smoke check and the benchmark's CPU-baseline leg.

Each function names the passage of the paper (arXiv 1803.03288) it follows;
the C file's header lists the readings taken where the paper is silent.
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tictac_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

PRIO_INF = np.iinfo(np.int32).max


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (``-O2``, no threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib: Optional[ctypes.CDLL] = None


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("oracle_find_dependencies", "oracle_update_properties", "oracle_tic",
                     "oracle_tac", "oracle_simulate"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what} failed with code {rc}" + (" (cycle)" if rc == -1 else ""))


def find_dependencies(n_ops: int, row_ptr, col_idx, recv_ids) -> np.ndarray:
    """Sec. 4.1, ``op.dep``: ``uint64 [n_ops][W]`` bitset of the recvs each op depends on
    directly or transitively (a recv's set holds itself)."""
    row_ptr, col_idx, recv_ids = _i32(row_ptr), _i32(col_idx), _i32(recv_ids)
    R = recv_ids.size
    W = (R + 63) // 64
    dep = np.zeros((n_ops, W), dtype=np.uint64)
    rc = _load().oracle_find_dependencies(ctypes.c_int(n_ops), _p(row_ptr), _p(col_idx), ctypes.c_int(R),
                                          _p(recv_ids), _p(dep))
    _check(rc, "oracle_find_dependencies")
    return dep


def update_properties(dep: np.ndarray, recv_ids, time, alive) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Sec. 4.1, Algorithm 1.  ``time [n_ops]`` by op id, ``alive [R]`` marks the
    outstanding recvs.  Returns ``(M [n_ops], P [R], Mplus [R])``."""
    dep = np.ascontiguousarray(dep, dtype=np.uint64)
    recv_ids, time = _i32(recv_ids), _f64(time)
    alive = np.ascontiguousarray(alive, dtype=np.uint8)
    n, R = dep.shape[0], recv_ids.size
    M, P, Mplus = np.zeros(n), np.zeros(R), np.zeros(R)
    rc = _load().oracle_update_properties(ctypes.c_int(n), ctypes.c_int(R), _p(dep), _p(recv_ids), _p(time),
                                          _p(alive), _p(M), _p(P), _p(Mplus))
    _check(rc, "oracle_update_properties")
    return M, P, Mplus


def tic(dep: np.ndarray, recv_ids) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Sec. 4.2, Algorithm 2.  Returns ``(prio, order, rank)``, all ``int32 [R]``:
    ``prio`` = M+ under the General Time Oracle (``PRIO_INF`` if none), ``order`` = recv
    indices sorted by ``(prio, index)``, ``rank`` its inverse."""
    dep = np.ascontiguousarray(dep, dtype=np.uint64)
    recv_ids = _i32(recv_ids)
    n, R = dep.shape[0], recv_ids.size
    prio, order, rank = (np.zeros(R, dtype=np.int32) for _ in range(3))
    rc = _load().oracle_tic(ctypes.c_int(n), ctypes.c_int(R), _p(dep), _p(recv_ids), _p(prio), _p(order), _p(rank))
    _check(rc, "oracle_tic")
    return prio, order, rank


def tac(dep: np.ndarray, recv_ids, op_time, recv_time, max_rounds: int = -1, comparator_mode: int = 0,
        alive0=None):
    """Sec. 4.3, Algorithm 3, for every row of ``op_time [B][N]`` / ``recv_time [B][R]``.
    ``alive0 [B][R]`` (optional) marks the recvs that are still outstanding when the loop starts
    (default: all of them, as the algorithm states); steps are then counted from that set.
    Returns ``(order, rank, sel_P, sel_Mplus)``, each ``[B][R]``."""
    dep = np.ascontiguousarray(dep, dtype=np.uint64)
    recv_ids, op_time, recv_time = _i32(recv_ids), _f64(op_time), _f64(recv_time)
    n, R = dep.shape[0], recv_ids.size
    B = recv_time.shape[0]
    assert op_time.shape == (B, n - R) and recv_time.shape == (B, R)
    a0 = None
    if alive0 is not None:
        a0 = np.ascontiguousarray(alive0, dtype=np.uint8)
        assert a0.shape == (B, R)
    order = np.full((B, R), -1, dtype=np.int32)
    rank = np.full((B, R), -1, dtype=np.int32)
    sel_P = np.full((B, R), np.nan)
    sel_Mplus = np.full((B, R), np.nan)
    rc = _load().oracle_tac(ctypes.c_int(n), ctypes.c_int(R), _p(dep), _p(recv_ids), ctypes.c_int(B), _p(op_time),
                            _p(recv_time), _p(a0), ctypes.c_int(max_rounds), ctypes.c_int(comparator_mode),
                            _p(order), _p(rank), _p(sel_P), _p(sel_Mplus))
    _check(rc, "oracle_tac")
    return order, rank, sel_P, sel_Mplus


def simulate(n_ops: int, row_ptr, col_idx, recv_ids, order, op_time, recv_time, pick_key=None):
    """Sec. 3.1-3.2 and 5.1: event-driven iteration on one compute device and one channel
    under a transfer order.  ``order`` is ``[R]`` (shared) or ``[B][R]``.
    Returns ``(makespan, E, U, L, S)``, each ``[B]``."""
    row_ptr, col_idx, recv_ids = _i32(row_ptr), _i32(col_idx), _i32(recv_ids)
    op_time, recv_time, order = _f64(op_time), _f64(recv_time), _i32(order)
    R = recv_ids.size
    B = recv_time.shape[0]
    assert op_time.shape == (B, n_ops - R) and recv_time.shape == (B, R)
    if order.ndim == 1:
        assert order.shape == (R,)
        stride = 0
    else:
        assert order.shape == (B, R)
        stride = R
    key = None if pick_key is None else _i32(pick_key)
    out = [np.zeros(B) for _ in range(5)]
    rc = _load().oracle_simulate(ctypes.c_int(n_ops), _p(row_ptr), _p(col_idx), ctypes.c_int(R), _p(recv_ids),
                                 ctypes.c_int(B), _p(order), ctypes.c_int(stride), _p(op_time), _p(recv_time),
                                 _p(key), *(_p(o) for o in out))
    _check(rc, "oracle_simulate")
    return tuple(out)


def simulate_channels(n_ops: int, row_ptr, col_idx, recv_ids, n_channels: int, channel_of_recv, order, op_time,
                      recv_time):
    """Sec. 4.1 / 5.1: the iteration of ``simulate`` with ``n_channels`` channels side by side; recv
    ``i`` uses channel ``channel_of_recv[i]`` and every channel serves its recvs in the order in
    which they appear in ``order``.  Returns ``(makespan, E, U, L, S)``, each ``[B]``."""
    row_ptr, col_idx, recv_ids = _i32(row_ptr), _i32(col_idx), _i32(recv_ids)
    op_time, recv_time, order, chan = _f64(op_time), _f64(recv_time), _i32(order), _i32(channel_of_recv)
    R = recv_ids.size
    B = recv_time.shape[0]
    assert op_time.shape == (B, n_ops - R) and recv_time.shape == (B, R) and chan.shape == (R,)
    if order.ndim == 1:
        assert order.shape == (R,)
        stride = 0
    else:
        assert order.shape == (B, R)
        stride = R
    out = [np.zeros(B) for _ in range(5)]
    rc = _load().oracle_simulate_channels(ctypes.c_int(n_ops), _p(row_ptr), _p(col_idx), ctypes.c_int(R),
                                          _p(recv_ids), ctypes.c_int(n_channels), _p(chan), ctypes.c_int(B),
                                          _p(order), ctypes.c_int(stride), _p(op_time), _p(recv_time),
                                          *(_p(o) for o in out))
    _check(rc, "oracle_simulate_channels")
    return tuple(out)


def simulate_sends(n_ops: int, row_ptr, col_idx, recv_ids, send_ids, order, op_time, recv_time, pick_key=None):
    """Sec. 2.2: the iteration of ``simulate`` with send ops (leaves of the graph) on an uplink that carries one
    transfer at a time, first come first served; the compute device picks the ready op of lowest ``pick_key``
    (default: lowest op id).  ``op_time`` holds a send's transfer time in its column.
    Returns ``(makespan, E, U, L, S)``, each ``[B]``."""
    row_ptr, col_idx, recv_ids, send_ids = _i32(row_ptr), _i32(col_idx), _i32(recv_ids), _i32(send_ids)
    op_time, recv_time, order = _f64(op_time), _f64(recv_time), _i32(order)
    R = recv_ids.size
    B = recv_time.shape[0]
    assert op_time.shape == (B, n_ops - R) and recv_time.shape == (B, R)
    if order.ndim == 1:
        assert order.shape == (R,)
        stride = 0
    else:
        assert order.shape == (B, R)
        stride = R
    key = None if pick_key is None else _i32(pick_key)
    out = [np.zeros(B) for _ in range(5)]
    rc = _load().oracle_simulate_sends(ctypes.c_int(n_ops), _p(row_ptr), _p(col_idx), ctypes.c_int(R), _p(recv_ids),
                                       ctypes.c_int(send_ids.size), _p(send_ids), ctypes.c_int(B), _p(order),
                                       ctypes.c_int(stride), _p(op_time), _p(recv_time), _p(key),
                                       *(_p(o) for o in out))
    _check(rc, "oracle_simulate_sends")
    return tuple(out)


def straggler(makespan, w: int) -> np.ndarray:
    """Sec. 6, Straggler Effect: per group of ``w`` consecutive samples, the longest wait of any
    worker over the iteration time, ``(max - min) / max`` of the group's makespans.
    Returns ``[B // w]``."""
    makespan = _f64(makespan)
    B = makespan.size
    out = np.zeros(B // w if w >= 1 else 0)
    rc = _load().oracle_straggler(ctypes.c_int(B), ctypes.c_int(w), _p(makespan), _p(out))
    _check(rc, "oracle_straggler")
    return out


def time_oracle_min(runs) -> np.ndarray:
    """Sec. 5, Time Oracle: the smallest of the measured runs of every op.  ``runs [K][n]`` -> ``[n]``."""
    runs = _f64(runs)
    assert runs.ndim == 2 and runs.shape[0] >= 1
    K, n = runs.shape
    out = np.zeros(n)
    rc = _load().oracle_time_oracle_min(ctypes.c_int(K), ctypes.c_longlong(n), _p(runs), _p(out))
    _check(rc, "oracle_time_oracle_min")
    return out



def order_search(n_ops: int, row_ptr, col_idx, recv_ids, order, moves, op_time, recv_time):
    """Sec. 3.1 / 4.3: every sample climbs from its start order through the proposed exchanges
    ``moves [n_moves][2]`` (positions of the order), keeping an exchange only when the makespan
    of ``simulate`` gets strictly smaller.  ``order`` is ``[R]`` (shared) or ``[B][R]``.
    Returns ``(best_order [B][R], best_makespan [B], start_makespan [B], n_accepted [B])``."""
    row_ptr, col_idx, recv_ids = _i32(row_ptr), _i32(col_idx), _i32(recv_ids)
    op_time, recv_time, order = _f64(op_time), _f64(recv_time), _i32(order)
    moves = _i32(moves).reshape(-1, 2)
    R = recv_ids.size
    B = recv_time.shape[0]
    assert op_time.shape == (B, n_ops - R) and recv_time.shape == (B, R)
    if order.ndim == 1:
        assert order.shape == (R,)
        stride = 0
    else:
        assert order.shape == (B, R)
        stride = R
    best = np.zeros((B, R), dtype=np.int32)
    m_best, m_start = np.zeros(B), np.zeros(B)
    n_acc = np.zeros(B, dtype=np.int32)
    rc = _load().oracle_order_search(ctypes.c_int(n_ops), _p(row_ptr), _p(col_idx), ctypes.c_int(R), _p(recv_ids),
                                     ctypes.c_int(B), _p(order), ctypes.c_int(stride), ctypes.c_int(moves.shape[0]),
                                     _p(moves), _p(op_time), _p(recv_time), _p(best), _p(m_best), _p(m_start),
                                     _p(n_acc))
    _check(rc, "oracle_order_search")
    return best, m_best, m_start, n_acc
