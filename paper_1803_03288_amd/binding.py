"""ctypes binding of ``libtictac.so`` (C ABI declared in ``include/tictac.h``).

Argument marshalling only: every step of the method runs in the library's HIP
kernels.  PyTorch is used for device memory (outputs are returned as CUDA tensors)
and for the current stream.  There is no CPU fallback: if the compiled library is
missing, importing a function from here raises.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtictac.so")

PRIO_INF = np.iinfo(np.int32).max

STATUS = {
    0: "TICTAC_OK", -1: "TICTAC_ERR_NULL", -2: "TICTAC_ERR_BAD_CSR", -3: "TICTAC_ERR_CYCLE",
    -4: "TICTAC_ERR_RECV_NOT_ROOT", -5: "TICTAC_ERR_DUP_RECV", -6: "TICTAC_ERR_BAD_ORDER",
    -7: "TICTAC_ERR_HIP", -8: "TICTAC_ERR_NO_MEM", -9: "TICTAC_ERR_UNSUPPORTED",
}

EXPORTS = (
    "tictac_build_deps", "tictac_dag_info", "tictac_dag_deps", "tictac_dag_copy_deps", "tictac_dag_recompute_deps",
    "tictac_dag_recompute_deps_batch", "tictac_dag_check_orders",
    "tictac_dag_free",
    "tictac_tic_priority", "tictac_tac_priority", "tictac_simulate", "tictac_tac_simulate",
    "tictac_tac_simulate_noalloc",
    "tictac_simulate_f32", "tictac_tac_simulate_f32",
    "tictac_simulate_channels", "tictac_simulate_sends", "tictac_straggler_effect", "tictac_time_oracle_min", "tictac_order_search",
    "tictac_last_error", "tictac_version",
)


class TicTacError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{STATUS.get(code, code)}: {message}")
        self.code = code


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (run ``python -m paper_1803_03288_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with paper_1803_03288_amd/build.py")
        L = ctypes.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(L, name).restype = ctypes.c_int
        L.tictac_last_error.restype = ctypes.c_char_p
        L.tictac_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise TicTacError(rc, lib().tictac_last_error().decode())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None or t.numel() == 0 else t.data_ptr())


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _np_ptr(a: np.ndarray) -> ctypes.c_void_p:
    return a.ctypes.data_as(ctypes.c_void_p)


class Dag:
    """Owner of a ``tictac_dag`` handle."""

    def __init__(self, handle: ctypes.c_void_p):
        self._h = handle
        vals = [ctypes.c_int32() for _ in range(5)]
        _check(lib().tictac_dag_info(self._h, *(ctypes.byref(v) for v in vals)))
        self.n_ops, self.n_recv, self.words, self.n_levels, self.n_classes = (v.value for v in vals)
        self.n_compute = self.n_ops - self.n_recv

    def deps(self) -> torch.Tensor:
        """op.dep as an int64 CUDA tensor ``[n_ops][W]`` (bit patterns of the uint64 words)."""
        out = torch.empty((self.n_ops, self.words), dtype=torch.int64, device="cuda")
        _check(lib().tictac_dag_copy_deps(self._h, _dev(out), _stream()))
        return out

    def deps_view(self) -> torch.Tensor:
        """The handle's own op.dep (``tictac_dag_deps``, borrowed) as an int64 CUDA tensor ``[n_ops][W]``: writes
        through it change the handle.  Valid until ``close``."""
        ptr = ctypes.c_void_p()
        _check(lib().tictac_dag_deps(self._h, ctypes.byref(ptr)))
        n = self.n_ops * self.words
        if n == 0 or not ptr.value:
            return torch.empty((self.n_ops, self.words), dtype=torch.int64, device="cuda")
        iface = {"shape": (self.n_ops, self.words), "typestr": "<i8", "data": (ptr.value, False), "version": 2,
                 "strides": None}
        holder = type("_Borrowed", (), {"__cuda_array_interface__": iface})()
        return torch.as_tensor(holder, device="cuda")

    def recompute_deps(self) -> None:
        """``tictac_dag_recompute_deps``: run the propagation kernel again (for timing)."""
        _check(lib().tictac_dag_recompute_deps(self._h, _stream()))

    def check_orders(self) -> None:
        """``tictac_dag_check_orders``: waits for the stream; raises ``TicTacError`` (TICTAC_ERR_BAD_ORDER) when an order
        given to a simulation or a search since the last call was no permutation of the recvs."""
        _check(lib().tictac_dag_check_orders(self._h, _stream()))

    def close(self) -> None:
        if self._h is not None:
            lib().tictac_dag_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def recompute_deps_batch(dags) -> None:
    """``tictac_dag_recompute_deps_batch``: the propagation kernel for several handles in one launch."""
    arr = (ctypes.c_void_p * len(dags))(*[d._h for d in dags])
    _check(lib().tictac_dag_recompute_deps_batch(arr, ctypes.c_int32(len(dags)), _stream()))


def build_deps(n_ops: int, row_ptr, col_idx, recv_ids) -> Dag:
    """``tictac_build_deps``: host predecessor CSR and recv ids in, handle out."""
    row_ptr, col_idx, recv_ids = _host_i32(row_ptr), _host_i32(col_idx), _host_i32(recv_ids)
    h = ctypes.c_void_p()
    _check(lib().tictac_build_deps(ctypes.c_int32(n_ops), _np_ptr(row_ptr), _np_ptr(col_idx),
                                   ctypes.c_int32(recv_ids.size), _np_ptr(recv_ids), _stream(), ctypes.byref(h)))
    return Dag(h)


def tic_priority(dag: Dag) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """``tictac_tic_priority``: ``(prio, order, rank)``, int32 CUDA tensors ``[R]``."""
    R = dag.n_recv
    prio, order, rank = (torch.empty(R, dtype=torch.int32, device="cuda") for _ in range(3))
    _check(lib().tictac_tic_priority(dag._h, _dev(prio), _dev(order), _dev(rank), _stream()))
    return prio, order, rank


def _check_times(dag: Dag, op_time: torch.Tensor, recv_time: torch.Tensor, allow_f32: bool = False) -> int:
    B = recv_time.shape[0]
    assert op_time.is_cuda and recv_time.is_cuda
    assert op_time.dtype == recv_time.dtype
    assert op_time.dtype == torch.float64 or (allow_f32 and op_time.dtype == torch.float32)
    assert op_time.is_contiguous() and recv_time.is_contiguous()
    assert tuple(op_time.shape) == (B, dag.n_compute), (tuple(op_time.shape), (B, dag.n_compute))
    assert tuple(recv_time.shape) == (B, dag.n_recv)
    return B


def tac_priority(dag: Dag, op_time: torch.Tensor, recv_time: torch.Tensor, want_rank: bool = True,
                 want_sel: bool = False):
    """``tictac_tac_priority``: ``(order, rank, sel_P, sel_Mplus)``, each ``[B][R]`` (None if not asked for)."""
    B = _check_times(dag, op_time, recv_time)
    R = dag.n_recv
    order = torch.empty((B, R), dtype=torch.int32, device="cuda")
    rank = torch.empty((B, R), dtype=torch.int32, device="cuda") if want_rank else None
    sel_P = torch.empty((B, R), dtype=torch.float64, device="cuda") if want_sel else None
    sel_M = torch.empty((B, R), dtype=torch.float64, device="cuda") if want_sel else None
    _check(lib().tictac_tac_priority(dag._h, ctypes.c_int32(B), _dev(op_time), _dev(recv_time), _dev(order),
                                     _dev(rank), _dev(sel_P), _dev(sel_M), _stream()))
    return order, rank, sel_P, sel_M


def simulate(dag: Dag, order: torch.Tensor, op_time: torch.Tensor, recv_time: torch.Tensor):
    """``tictac_simulate`` (``tictac_simulate_f32`` for float32 timing arrays): ``(makespan, eff, U, L, S)``,
    float64 CUDA tensors ``[B]``.  ``order`` is int32 ``[R]`` (shared) or ``[B][R]``."""
    B = _check_times(dag, op_time, recv_time, allow_f32=True)
    R = dag.n_recv
    assert order.is_cuda and order.dtype == torch.int32 and order.is_contiguous()
    if order.dim() == 1:
        assert order.shape[0] == R
        stride = 0
    else:
        assert tuple(order.shape) == (B, R)
        stride = R
    out = [torch.empty(B, dtype=torch.float64, device="cuda") for _ in range(5)]
    fn = lib().tictac_simulate_f32 if op_time.dtype == torch.float32 else lib().tictac_simulate
    _check(fn(dag._h, ctypes.c_int32(B), _dev(order), ctypes.c_int32(stride), _dev(op_time), _dev(recv_time),
              *(_dev(o) for o in out), _stream()))
    return tuple(out)


def simulate_channels(dag: Dag, n_channels: int, channel_of_recv, order: torch.Tensor, op_time: torch.Tensor,
                      recv_time: torch.Tensor):
    """``tictac_simulate_channels``: ``(makespan, eff, U, L, S)``, float64 CUDA tensors ``[B]``.
    ``channel_of_recv`` is a host int32 array ``[R]``; ``order`` is int32 ``[R]`` or ``[B][R]``."""
    B = _check_times(dag, op_time, recv_time)
    R = dag.n_recv
    chan = np.ascontiguousarray(channel_of_recv, dtype=np.int32)
    assert chan.shape == (R,)
    assert order.is_cuda and order.dtype == torch.int32 and order.is_contiguous()
    if order.dim() == 1:
        assert order.shape[0] == R
        stride = 0
    else:
        assert tuple(order.shape) == (B, R)
        stride = R
    out = [torch.empty(B, dtype=torch.float64, device="cuda") for _ in range(5)]
    _check(lib().tictac_simulate_channels(dag._h, ctypes.c_int32(B), ctypes.c_int32(n_channels),
                                          chan.ctypes.data_as(ctypes.c_void_p), _dev(order), ctypes.c_int32(stride),
                                          _dev(op_time), _dev(recv_time), *(_dev(o) for o in out), _stream()))
    return tuple(out)


def time_oracle_min(runs: torch.Tensor) -> torch.Tensor:
    """``tictac_time_oracle_min``: ``runs`` float64 CUDA ``[K][...]`` -> the minimum over the K runs."""
    assert runs.is_cuda and runs.dtype == torch.float64 and runs.is_contiguous() and runs.dim() >= 2
    K = runs.shape[0]
    out = torch.empty(runs.shape[1:], dtype=torch.float64, device="cuda")
    _check(lib().tictac_time_oracle_min(ctypes.c_int32(K), ctypes.c_int64(out.numel()), _dev(runs), _dev(out), _stream()))
    return out


def simulate_sends(dag: Dag, send_ids, order: torch.Tensor, op_time: torch.Tensor, recv_time: torch.Tensor):
    """``tictac_simulate_sends``: ``(makespan, eff, U, L, S)``, float64 CUDA tensors ``[B]``.  ``send_ids`` is a host
    int32 array of op ids (leaves of the graph); ``order`` is int32 ``[R]`` or ``[B][R]``."""
    B = _check_times(dag, op_time, recv_time)
    R = dag.n_recv
    sends = np.ascontiguousarray(send_ids, dtype=np.int32)
    assert sends.ndim == 1
    assert order.is_cuda and order.dtype == torch.int32 and order.is_contiguous()
    if order.dim() == 1:
        assert order.shape[0] == R
        stride = 0
    else:
        assert tuple(order.shape) == (B, R)
        stride = R
    out = [torch.empty(B, dtype=torch.float64, device=recv_time.device) for _ in range(5)]
    _check(lib().tictac_simulate_sends(dag._h, ctypes.c_int32(B), ctypes.c_int32(sends.size),
                                       sends.ctypes.data_as(ctypes.c_void_p), _dev(order), ctypes.c_int32(stride),
                                       _dev(op_time), _dev(recv_time), *(_dev(o) for o in out), _stream()))
    return tuple(out)


def order_search(dag: Dag, order: torch.Tensor, moves: torch.Tensor, op_time: torch.Tensor, recv_time: torch.Tensor):
    """``tictac_order_search``: ``order`` int32 CUDA ``[R]`` or ``[B][R]`` (start orders), ``moves`` int32
    CUDA ``[n_moves][2]``.  Returns ``(best_order [B][R], best_makespan, start_makespan, n_accepted)``."""
    B = _check_times(dag, op_time, recv_time)
    R = dag.n_recv
    assert order.is_cuda and order.dtype == torch.int32 and order.is_contiguous()
    assert moves.is_cuda and moves.dtype == torch.int32 and moves.is_contiguous()
    assert moves.dim() == 2 and moves.shape[1] == 2
    if order.dim() == 1:
        assert order.shape == (R,)
        stride = 0
    else:
        assert order.shape == (B, R)
        stride = R
    best = torch.empty((B, R), dtype=torch.int32, device="cuda")
    m_best = torch.empty(B, dtype=torch.float64, device="cuda")
    m_start = torch.empty(B, dtype=torch.float64, device="cuda")
    n_acc = torch.empty(B, dtype=torch.int32, device="cuda")
    _check(lib().tictac_order_search(dag._h, ctypes.c_int32(B), _dev(order), ctypes.c_int32(stride),
                                     ctypes.c_int32(moves.shape[0]), _dev(moves), _dev(op_time), _dev(recv_time),
                                     _dev(best), _dev(m_best), _dev(m_start), _dev(n_acc), _stream()))
    return best, m_best, m_start, n_acc


def straggler_effect(makespan: torch.Tensor, w: int) -> torch.Tensor:
    """``tictac_straggler_effect``: float64 CUDA tensor ``[B // w]``."""
    assert makespan.is_cuda and makespan.dtype == torch.float64 and makespan.is_contiguous() and makespan.dim() == 1
    B = makespan.shape[0]
    out = torch.empty(B // w if w >= 1 else 0, dtype=torch.float64, device="cuda")
    _check(lib().tictac_straggler_effect(ctypes.c_int32(B), ctypes.c_int32(w), _dev(makespan), _dev(out), _stream()))
    return out


def tac_simulate(dag: Dag, op_time: torch.Tensor, recv_time: torch.Tensor, want_rank: bool = False,
                 want_sel: bool = False):
    """``tictac_tac_simulate`` (``tictac_tac_simulate_f32`` for float32 timing arrays): TAC and the iteration
    under its order in one pass.  Returns ``(order, rank, sel_P, sel_Mplus, makespan, eff, U, L, S)``."""
    B = _check_times(dag, op_time, recv_time, allow_f32=True)
    R = dag.n_recv
    # (one allocation per dtype: the outputs are rows of two blocks)
    ints = torch.empty((2 if want_rank else 1, B, R), dtype=torch.int32, device="cuda")
    order, rank = ints[0], (ints[1] if want_rank else None)
    sel_P = torch.empty((B, R), dtype=torch.float64, device="cuda") if want_sel else None
    sel_M = torch.empty((B, R), dtype=torch.float64, device="cuda") if want_sel else None
    out = torch.empty((5, B), dtype=torch.float64, device="cuda").unbind(0)
    fn = lib().tictac_tac_simulate_f32 if op_time.dtype == torch.float32 else lib().tictac_tac_simulate
    _check(fn(dag._h, ctypes.c_int32(B), _dev(op_time), _dev(recv_time), _dev(order), _dev(rank), _dev(sel_P),
              _dev(sel_M), *(_dev(o) for o in out), _stream()))
    return (order, rank, sel_P, sel_M) + tuple(out)


def tac_simulate_noalloc(dag: Dag, op_time: torch.Tensor, recv_time: torch.Tensor, out: Tuple[torch.Tensor, ...]):
    """``tictac_tac_simulate_noalloc``: the call that allocates nothing.  ``out`` are the caller's tensors
    ``(order [B][R] int32, rank [B][R] int32 or None, makespan, eff, U, L, S [B] float64)``; they are
    written and returned."""
    B = _check_times(dag, op_time, recv_time)
    order, rank, m, e, U, L, S = out
    assert order.dtype == torch.int32 and tuple(order.shape) == (B, dag.n_recv) and order.is_contiguous()
    for x in (m, e, U, L, S):
        assert x.dtype == torch.float64 and tuple(x.shape) == (B,) and x.is_contiguous()
    _check(lib().tictac_tac_simulate_noalloc(dag._h, ctypes.c_int32(B), _dev(op_time), _dev(recv_time), _dev(order),
                                             _dev(rank), _dev(m), _dev(e), _dev(U), _dev(L), _dev(S), _stream()))
    return out


def version() -> str:
    return lib().tictac_version().decode()
