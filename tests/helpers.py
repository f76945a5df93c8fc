"""Independent helpers for the tests: second implementations and brute force written
directly from definitions (numpy / pure Python), a golden-file reader, and the
time-row assembly shared by the oracle pins and the GPU parity tests.  None of this
is used by the library or by the oracle."""

from __future__ import annotations

import itertools
import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name: str) -> Dict[str, np.ndarray]:
    out: Dict[str, np.ndarray] = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=", 1)
            out[k.strip()] = np.array([float(x) for x in v.split()], dtype=np.float64)
    return out


def bits_of_row(row: np.ndarray) -> List[int]:
    out = []
    for w, word in enumerate(row):
        word = int(word)
        for b in range(64):
            if (word >> b) & 1:
                out.append(w * 64 + b)
    return out


def dep_bool(dep: np.ndarray, R: int) -> np.ndarray:
    """[n][R] boolean matrix of a bitset matrix."""
    n, W = dep.shape
    if W == 0:
        return np.zeros((n, 0), dtype=bool)
    b = np.unpackbits(dep.view(np.uint8).reshape(n, W * 8), axis=1, bitorder="little")
    return b[:, :R].astype(bool)


def recv_ancestors_bfs(dag) -> np.ndarray:
    """[n][R] reachability by a breadth-first search from every op over predecessor
    edges (brute force, only for small graphs)."""
    n, R = dag.n_ops, dag.n_recv
    ri = {int(v): i for i, v in enumerate(dag.recv_ids)}
    out = np.zeros((n, R), dtype=bool)
    for v in range(n):
        seen = {v}
        frontier = [v]
        while frontier:
            nxt = []
            for x in frontier:
                if x in ri:
                    out[v, ri[x]] = True
                for p in dag.col_idx[dag.row_ptr[x]:dag.row_ptr[x + 1]]:
                    p = int(p)
                    if p not in seen:
                        seen.add(p)
                        nxt.append(p)
            frontier = nxt
    return out


def full_time_row(dag, op_row: np.ndarray, recv_row: np.ndarray) -> np.ndarray:
    """Time(op) by op id from one row of op_time and recv_time."""
    t = np.zeros(dag.n_ops)
    t[dag.compute_ids()] = op_row
    t[dag.recv_ids] = recv_row
    return t


def closed_form_makespan(depb: np.ndarray, dag, order: np.ndarray, op_time: np.ndarray,
                         recv_time: np.ndarray) -> np.ndarray:
    """Makespan of every sample from the recv-ancestor matrix alone.

    With one channel that never waits (recvs are roots) transfer k (1-based) ends at
    F_k = sum of the first k transfer times.  A compute op can start no earlier than
    F_kappa, kappa = the last position among the recvs it depends on (0 if none).  A
    work-conserving single device then finishes at  max_k (F_k + S_k),  S_k = total time
    of the compute ops with kappa >= k, and the iteration ends at the later of that and
    F_R.  `order` is [R] or [B][R]."""
    B = recv_time.shape[0]
    R = dag.n_recv
    comp = dag.compute_ids()
    dc = depb[comp]                                   # [N][R]
    order = np.asarray(order)
    per_sample = order.ndim == 2
    out = np.zeros(B)
    for b in range(B):
        o = order[b] if per_sample else order
        pos = np.zeros(R, dtype=np.int64)
        pos[o] = np.arange(1, R + 1)
        kappa = (dc * pos[None, :]).max(axis=1) if R else np.zeros(len(comp), dtype=np.int64)
        F = np.concatenate([[0.0], np.cumsum(recv_time[b][o])])
        A = np.bincount(kappa, weights=op_time[b], minlength=R + 1)
        S = np.cumsum(A[::-1])[::-1]
        out[b] = max((F + S).max(), F[-1])
    return out


def all_orders(R: int) -> np.ndarray:
    return np.array(list(itertools.permutations(range(R))), dtype=np.int32).reshape(-1, R)


def oracle_tac_rows(dep, recv_ids, op, rv, threads: int = 8, **kw):
    """``oracle.tac`` on the rows of ``op`` / ``rv``, the rows dealt to a few host threads (the
    oracle itself is single-threaded and the samples are independent; ctypes releases the
    interpreter lock during the call).  ``alive0`` in ``kw`` is split along with the rows."""
    import oracle
    B = rv.shape[0]
    threads = max(1, min(threads, B))
    bounds = np.linspace(0, B, threads + 1).astype(int)
    alive0 = kw.pop("alive0", None)

    def part(i):
        lo, hi = bounds[i], bounds[i + 1]
        a0 = None if alive0 is None else alive0[lo:hi]
        return oracle.tac(dep, recv_ids, op[lo:hi], rv[lo:hi], alive0=a0, **kw)

    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(part, range(threads)))
    return tuple(np.concatenate([p[j] for p in parts], axis=0) for j in range(4))


def oracle_rounds_after_prefix(dep, recv_ids, op_row, rv_row, order_row, ks, threads: int = 8):
    """For every k in ``ks``: the recv that Algorithm 3 selects, with its P and M+, when the recvs
    ``order_row[:k]`` have been removed, i.e. round k of the sample as the oracle sees it after the
    given prefix.  Returns ``(selected [len(ks)], P, Mplus)``."""
    R = order_row.shape[0]
    ks = list(ks)
    alive0 = np.ones((len(ks), R), dtype=np.uint8)
    for j, k in enumerate(ks):
        alive0[j, order_row[:k]] = 0
    op = np.repeat(op_row[None, :], len(ks), axis=0)
    rv = np.repeat(rv_row[None, :], len(ks), axis=0)
    o, _, sP, sM = oracle_tac_rows(dep, recv_ids, op, rv, threads=threads, alive0=alive0, max_rounds=1)
    sel = o[:, 0]
    rows = np.arange(len(ks))
    return sel, sP[rows, sel], sM[rows, sel]


def tac_order_up_to_near_ties(oracle, dag, dep, op_row, rv_row, got, tol=1e-12, max_restarts=64):
    """Checks one TAC order computed in floating point on times that are not quantised.

    Where `got` equals the oracle's order nothing is to show.  At the first step where they differ the
    oracle's round (Algorithm 1 on the recvs still outstanding) must call it a near tie: no outstanding
    recv precedes the one `got` chose by more than `tol` relative in the comparator's min-terms
    (Sec. 4.3, Case 1), nor, where those are equal bit for bit, in M+ (Case 2), nor, where M+ is equal bit
    for bit too, by its smaller index.  The oracle is then
    continued from the prefix of `got` (its start-set argument) and the rest compared the same way.
    Returns the number of near ties met; raises AssertionError on any other difference."""
    R = dag.n_recv
    got = np.asarray(got)
    assert np.array_equal(np.sort(got), np.arange(R)), "not a permutation"
    t = full_time_row(dag, op_row, rv_row)
    alive = np.ones(R, dtype=np.uint8)
    k, near = 0, 0
    while k < R:
        exp = oracle.tac(dep, dag.recv_ids, op_row[None], rv_row[None], alive0=alive[None])[0][0][: R - k]
        diff = np.nonzero(exp != got[k:])[0]
        if diff.size == 0:
            break
        j = k + int(diff[0])
        alive[got[k:j]] = 0
        M, P, Mp = oracle.update_properties(dep, dag.recv_ids, t, alive)
        Mr = M[dag.recv_ids]
        g = int(got[j])
        for c in np.nonzero(alive)[0]:
            if c == g:
                continue
            x, y = min(P[g], Mr[c]), min(P[c], Mr[g])       # c before g iff x < y
            scale = max(abs(x), abs(y))
            assert not (x < y - tol * scale), (
                f"step {j}: recv {c} precedes the chosen recv {g} outright: {x!r} < {y!r}")
            if x == y:
                assert not (Mp[c] < Mp[g] - tol * max(abs(Mp[c]), abs(Mp[g]))), (
                    f"step {j}: equal min-terms and recv {c} has the smaller M+: {Mp[c]!r} < {Mp[g]!r}")
                assert not (Mp[c] == Mp[g] and c < g), (
                    f"step {j}: recvs {c} and {g} tie in every term and the smaller index goes first")
        near += 1
        assert near <= max_restarts, "too many near ties for one sample"
        alive[g] = 0
        k = j + 1
    return near


def tick_simulate_sends(dag, send_ids, order, op_row, recv_row):
    """The iteration with send ops, simulated tick by tick for whole-number durations (a second
    implementation for small cases; nothing in it is event-driven).  At every tick t: transfers and ops
    whose remaining time is zero complete, which may make ops ready; the compute device, when idle, starts
    the ready compute op of lowest id; the uplink, when idle, starts the send that was requested first
    (lowest id among those of one tick); the downlink serves the recvs back to back in `order`.  All of
    that is repeated within the tick until nothing changes (durations of zero), then one tick passes.
    Returns the makespan."""
    n = dag.n_ops
    t_of = full_time_row(dag, op_row, recv_row).astype(np.int64)
    assert np.array_equal(t_of, full_time_row(dag, op_row, recv_row)), "whole numbers only"
    is_recv = np.zeros(n, dtype=bool)
    is_recv[dag.recv_ids] = True
    is_send = np.zeros(n, dtype=bool)
    is_send[np.asarray(send_ids, dtype=np.int64)] = True
    preds = [list(map(int, dag.col_idx[dag.row_ptr[v]:dag.row_ptr[v + 1]])) for v in range(n)]
    done = np.zeros(n, dtype=bool)
    started = np.zeros(n, dtype=bool)
    requested_at = {}
    down = [int(dag.recv_ids[i]) for i in order]
    down_k, down_left = 0, (int(t_of[down[0]]) if down else 0)
    running, run_left = -1, 0
    sending, send_left = -1, 0
    t, last = 0, 0
    while not done.all():
        changed = True
        while changed:
            changed = False
            if down_k < len(down) and down_left == 0:
                done[down[down_k]] = True
                down_k += 1
                down_left = int(t_of[down[down_k]]) if down_k < len(down) else 0
                last, changed = t, True
            if running >= 0 and run_left == 0:
                done[running], running, last, changed = True, -1, t, True
            if sending >= 0 and send_left == 0:
                done[sending], sending, last, changed = True, -1, t, True
            ready = [v for v in range(n) if not is_recv[v] and not started[v] and all(done[u] for u in preds[v])]
            for v in ready:
                if is_send[v] and v not in requested_at:
                    requested_at[v] = t
            if running < 0:
                cand = [v for v in ready if not is_send[v]]
                if cand:
                    running = min(cand)
                    started[running], run_left, changed = True, int(t_of[running]), True
            if sending < 0:
                cand = [v for v in requested_at if not started[v]]
                if cand:
                    sending = min(cand, key=lambda v: (requested_at[v], v))
                    started[sending], send_left, changed = True, int(t_of[sending]), True
        if done.all():
            break
        t += 1
        if down_k < len(down):
            down_left -= 1
        if running >= 0:
            run_left -= 1
        if sending >= 0:
            send_left -= 1
        assert t < 10**6, "stuck"
    return last
