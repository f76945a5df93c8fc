"""Pins of the CPU oracle against what the paper and the mathematics fix: the worked
examples of the paper (tests/golden), closed forms, invariants, special cases that
reduce to textbook results (Johnson's rule for the two-machine flow shop) and brute
force on tiny inputs.  No GPU is involved."""

import numpy as np
import pytest

import oracle
from paper_1803_03288_amd import workloads as wl

from helpers import (all_orders, bits_of_row, closed_form_makespan, dep_bool, full_time_row,
                     read_golden, recv_ancestors_bfs)


def deps(d):
    return oracle.find_dependencies(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)


def sim(d, order, op, rv, key=None):
    return oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, order, op, rv, key)


def rand_times(rng, B, n, lo=1, hi=2000):
    """Random multiples of 2**-30 s (exact sums)."""
    return rng.integers(lo, hi, size=(B, n)).astype(np.float64) * wl.QUANTUM * 1024


# --------------------------------------------------------------------------
# worked examples printed in the paper
# --------------------------------------------------------------------------

def test_fig1_toy_graph_values():
    g = read_golden("fig1_toy.txt")
    d = wl.toy_dag()
    dep = deps(d)
    op1, op2 = d.compute_ids()
    assert bits_of_row(dep[op1]) == list(g["dep_op1"].astype(int))
    assert bits_of_row(dep[op2]) == list(g["dep_op2"].astype(int))
    rv, op = g["recv_time"][None, :], g["op_time"][None, :]
    t = full_time_row(d, op[0], rv[0])
    M, P, Mplus = oracle.update_properties(dep, d.recv_ids, t, np.ones(2, dtype=np.uint8))
    assert M[op1] == g["M_op1"][0] and M[op2] == g["M_op2"][0]
    assert M[d.recv_ids[0]] == rv[0, 0] and M[d.recv_ids[1]] == rv[0, 1]    # recv.M = Time(recv)
    np.testing.assert_array_equal(P, g["P"])
    np.testing.assert_array_equal(Mplus, g["Mplus"])
    order, rank, sel_P, sel_Mplus = oracle.tac(dep, d.recv_ids, op, rv)
    np.testing.assert_array_equal(order[0], g["tac_order"].astype(int))
    np.testing.assert_array_equal(rank[0], [0, 1])
    m01, e01, U, L, S = sim(d, np.array([0, 1]), op, rv)
    m10, e10, _, _, _ = sim(d, np.array([1, 0]), op, rv)
    assert m01[0] == g["makespan_order_0_1"][0] and m10[0] == g["makespan_order_1_0"][0]
    assert U[0] == g["U"][0] and L[0] == g["L"][0] and S[0] == g["S"][0]
    assert e01[0] == pytest.approx(g["E_order_0_1"][0], rel=1e-15)
    assert e10[0] == g["E_order_1_0"][0]


def test_printed_comparator_listing_contradicts_toy_example():
    """The comparator as its listing prints it sends recv2 first on the toy graph,
    against Sec. 2.2; the derived pairwise rule (the oracle's reading) does not."""
    g = read_golden("fig1_toy.txt")
    d = wl.toy_dag()
    dep = deps(d)
    rv, op = g["recv_time"][None, :], g["op_time"][None, :]
    good = oracle.tac(dep, d.recv_ids, op, rv, comparator_mode=0)[0][0]
    printed = oracle.tac(dep, d.recv_ids, op, rv, comparator_mode=1)[0][0]
    assert list(good) == [0, 1] and list(printed) == [1, 0]


def test_case2_graph_values():
    g = read_golden("case2.txt")
    d = wl.case2_dag()
    dep = deps(d)
    rv, op = g["recv_time"][None, :], g["op_time"][None, :]
    t = full_time_row(d, op[0], rv[0])
    M, P, Mplus = oracle.update_properties(dep, d.recv_ids, t, np.ones(4, dtype=np.uint8))
    np.testing.assert_array_equal(P, g["P_round0"])
    np.testing.assert_array_equal(Mplus, g["Mplus_round0"])
    assert Mplus[0] == Mplus[1] == rv[0, 0] + rv[0, 1] < Mplus[2] < Mplus[3]
    prio, tic_order, _ = oracle.tic(dep, d.recv_ids)
    np.testing.assert_array_equal(prio, g["tic_prio"].astype(int))
    np.testing.assert_array_equal(tic_order, [0, 1, 2, 3])
    order, rank, sel_P, sel_Mplus = oracle.tac(dep, d.recv_ids, op, rv)
    np.testing.assert_array_equal(order[0], g["tac_order"].astype(int))
    np.testing.assert_array_equal(sel_P[0], g["sel_P"])
    np.testing.assert_array_equal(sel_Mplus[0], g["sel_Mplus"])
    m, e, U, L, S = sim(d, order[0], op, rv)
    assert m[0] == g["makespan"][0] and U[0] == g["U"][0] and L[0] == g["L"][0]
    assert e[0] == pytest.approx(g["E"][0], rel=1e-15)


def test_case1_two_job_makespan_formula_and_pairwise_rule():
    """Sec. 4.3 Case 1: Makespan(A->B) = M_A + max{P_A, M_B} + P_B, and A goes first
    iff min{P_B, M_A} < min{P_A, M_B}."""
    d = wl.independent_jobs_dag(2)
    dep = deps(d)
    rng = np.random.default_rng(11)
    B = 400
    rv, op = rand_times(rng, B, 2, 1, 50), rand_times(rng, B, 2, 1, 50)
    MA, MB, PA, PB = rv[:, 0], rv[:, 1], op[:, 0], op[:, 1]
    mab = sim(d, np.array([0, 1]), op, rv)[0]
    mba = sim(d, np.array([1, 0]), op, rv)[0]
    np.testing.assert_array_equal(mab, MA + np.maximum(PA, MB) + PB)
    np.testing.assert_array_equal(mba, MB + np.maximum(PB, MA) + PA)
    order = oracle.tac(dep, d.recv_ids, op, rv)[0]
    a_first = np.minimum(PB, MA) < np.minimum(PA, MB)
    b_first = np.minimum(PA, MB) < np.minimum(PB, MA)
    assert a_first.sum() > 50 and b_first.sum() > 50
    assert (order[a_first, 0] == 0).all() and (order[b_first, 0] == 1).all()
    # the rule is the makespan comparison
    assert ((mab < mba) == a_first).all()
    # TAC never picks the strictly worse order; the printed listing does
    chosen = np.where(order[:, 0] == 0, mab, mba)
    assert (chosen == np.minimum(mab, mba)).all()
    printed = oracle.tac(dep, d.recv_ids, op, rv, comparator_mode=1)[0]
    worse = np.where(printed[:, 0] == 0, mab, mba)
    assert (worse > np.minimum(mab, mba)).any()


# --------------------------------------------------------------------------
# dependency sets
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_dependencies_equal_bfs_reachability(seed):
    d = wl.layered_dag(seed, levels=6, width=5, fan_in=(1, 3), back=2, n_recv=70, attach=(1, 3))
    dep = deps(d)
    assert dep.shape == (d.n_ops, 2)
    np.testing.assert_array_equal(dep_bool(dep, d.n_recv), recv_ancestors_bfs(d))
    # padding bits beyond R stay clear
    assert (dep[:, 1] >> np.uint64(70 - 64)).max() == 0


def test_dependencies_monotone_along_edges_and_relabel():
    d = wl.layered_dag(5, levels=7, width=6, fan_in=(1, 3), back=3, n_recv=20, attach=(1, 4))
    dep = deps(d)
    for v in range(d.n_ops):
        for u in d.col_idx[d.row_ptr[v]:d.row_ptr[v + 1]]:
            assert ((dep[u] & ~dep[v]) == 0).all()
    d2, new_id = wl.relabel(d, 3)
    dep2 = deps(d2)
    np.testing.assert_array_equal(dep2[new_id], dep)


def test_cycle_is_reported():
    row_ptr = np.array([0, 0, 2, 3], dtype=np.int32)      # op1 <- {recv0, op2}; op2 <- {op1}
    col_idx = np.array([0, 2, 1], dtype=np.int32)
    with pytest.raises(RuntimeError):
        oracle.find_dependencies(3, row_ptr, col_idx, np.array([0], dtype=np.int32))


def test_chain_dependencies_and_priorities():
    """Layer-by-layer model: the priority order must equal the consumption order."""
    R = 9
    d = wl.chain_dag(R)
    dep = deps(d)
    comp = d.compute_ids()
    for k in range(R):
        assert bits_of_row(dep[comp[k]]) == list(range(k + 1))
    prio, order, rank = oracle.tic(dep, d.recv_ids)
    np.testing.assert_array_equal(prio, [2, 2] + list(range(3, R + 1)))
    np.testing.assert_array_equal(order, np.arange(R))
    rng = np.random.default_rng(5)
    rv, op = rand_times(rng, 64, R), rand_times(rng, 64, R)
    tac_order = oracle.tac(dep, d.recv_ids, op, rv)[0]
    assert (tac_order == np.arange(R)[None, :]).all()


# --------------------------------------------------------------------------
# TIC
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 7])
def test_tic_is_mplus_under_general_time_oracle(seed):
    d = wl.layered_dag(seed, levels=6, width=6, fan_in=(1, 3), back=2, n_recv=30, attach=(1, 3))
    dep = deps(d)
    t = np.zeros(d.n_ops)
    t[d.recv_ids] = 1.0
    M, P, Mplus = oracle.update_properties(dep, d.recv_ids, t, np.ones(d.n_recv, dtype=np.uint8))
    prio, order, rank = oracle.tic(dep, d.recv_ids)
    assert (P == 0).all()
    expect = np.where(np.isinf(Mplus), oracle.PRIO_INF, Mplus).astype(np.int64)
    np.testing.assert_array_equal(prio, expect)
    # definition by brute force: min size of a dependency set that holds the recv and another
    db = recv_ancestors_bfs(d)
    comp = d.compute_ids()
    cnt = db[comp].sum(axis=1)
    for i in range(d.n_recv):
        c = cnt[db[comp, i] & (cnt > 1)]
        assert prio[i] == (c.min() if c.size else oracle.PRIO_INF)
    # order = stable sort, rank = inverse
    np.testing.assert_array_equal(order, np.argsort(prio, kind="stable"))
    np.testing.assert_array_equal(rank[order], np.arange(d.n_recv))


def test_single_recv_has_no_finite_priority():
    d = wl.chain_dag(1)
    dep = deps(d)
    prio, order, rank = oracle.tic(dep, d.recv_ids)
    assert prio[0] == oracle.PRIO_INF and order[0] == 0 and rank[0] == 0


# --------------------------------------------------------------------------
# simulation: closed form, bounds, pick-rule invariance, degenerate graphs
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_simulation_equals_closed_form_and_is_pick_rule_invariant(seed):
    d = wl.layered_dag(seed, levels=8, width=6, fan_in=(1, 3), back=3, n_recv=12, attach=(1, 3))
    dep = deps(d)
    depb = dep_bool(dep, d.n_recv)
    rng = np.random.default_rng(seed)
    B = 40
    rv, op = rand_times(rng, B, d.n_recv), rand_times(rng, B, d.n_compute)
    op[rng.random(op.shape) < 0.15] = 0.0           # zero-duration ops
    rv[rng.random(rv.shape) < 0.10] = 0.0
    orders = np.stack([rng.permutation(d.n_recv) for _ in range(B)]).astype(np.int32)
    m, e, U, L, S = sim(d, orders, op, rv)
    np.testing.assert_array_equal(m, closed_form_makespan(depb, d, orders, op, rv))
    for key in (np.arange(d.n_ops)[::-1].copy(), rng.permutation(d.n_ops)):
        m2 = sim(d, orders, op, rv, key)[0]
        np.testing.assert_array_equal(m2, m)
    np.testing.assert_array_equal(U, op.sum(axis=1) + rv.sum(axis=1))
    np.testing.assert_array_equal(L, np.maximum(op.sum(axis=1), rv.sum(axis=1)))
    assert (L <= m).all() and (m <= U).all()
    assert (e >= 0).all() and (e <= 1).all()
    ok = U > L
    np.testing.assert_allclose(e[ok], ((U - m) / (U - L))[ok], rtol=1e-15)
    np.testing.assert_allclose(S[ok], ((U - L) / L)[ok], rtol=1e-15)
    # shared order = the same order for every sample
    m3 = sim(d, orders[0], op, rv)[0]
    np.testing.assert_array_equal(m3, closed_form_makespan(depb, d, orders[0], op, rv))


def test_no_recvs():
    d = wl.no_recv_dag(17)
    dep = deps(d)
    assert dep.shape == (17, 0)
    rng = np.random.default_rng(0)
    op = rand_times(rng, 5, 17)
    rv = np.zeros((5, 0))
    prio, order, rank = oracle.tic(dep, d.recv_ids)
    assert order.size == 0
    o = oracle.tac(dep, d.recv_ids, op, rv)[0]
    assert o.shape == (5, 0)
    m, e, U, L, S = sim(d, np.zeros(0, dtype=np.int32), op, rv)
    np.testing.assert_array_equal(m, op.sum(axis=1))
    np.testing.assert_array_equal(U, m)
    np.testing.assert_array_equal(L, m)
    assert (e == 1).all() and (S == 0).all()


def test_all_recvs_at_the_root_gives_zero_efficiency():
    R = 5
    d = wl.funnel_dag(R, 6)
    dep = deps(d)
    assert (dep_bool(dep, R)[d.compute_ids()]).all()
    prio, order, _ = oracle.tic(dep, d.recv_ids)
    assert (prio == R).all() and (order == np.arange(R)).all()
    rng = np.random.default_rng(1)
    perms = all_orders(R)
    rv = np.repeat(rand_times(rng, 1, R), len(perms), axis=0)
    op = np.repeat(rand_times(rng, 1, 6), len(perms), axis=0)
    m, e, U, L, S = sim(d, perms, op, rv)
    np.testing.assert_array_equal(m, U)
    assert (e == 0).all()
    tac_order = oracle.tac(dep, d.recv_ids, op[:1], rv[:1])[0][0]
    np.testing.assert_array_equal(tac_order, np.arange(R))


def test_unused_recvs_and_free_compute_give_full_overlap():
    # 3 recvs without consumers, 4 chained compute ops without recv dependencies
    row_ptr = np.array([0, 0, 0, 0, 0, 1, 2, 3], dtype=np.int32)
    col_idx = np.array([3, 4, 5], dtype=np.int32)
    recv_ids = np.array([0, 1, 2], dtype=np.int32)
    rng = np.random.default_rng(2)
    rv, op = rand_times(rng, 6, 3), rand_times(rng, 6, 4)
    m, e, U, L, S = oracle.simulate(7, row_ptr, col_idx, recv_ids, np.array([2, 0, 1]), op, rv)
    np.testing.assert_array_equal(m, L)
    assert (e == 1).all()
    dep = oracle.find_dependencies(7, row_ptr, col_idx, recv_ids)
    prio, order, _ = oracle.tic(dep, recv_ids)
    assert (prio == oracle.PRIO_INF).all() and list(order) == [0, 1, 2]
    tac_order, _, sel_P, sel_Mplus = oracle.tac(dep, recv_ids, op, rv)
    assert (tac_order == np.arange(3)).all() and (sel_P == 0).all() and np.isinf(sel_Mplus).all()


# --------------------------------------------------------------------------
# Johnson's rule and brute force over all transfer orders
# --------------------------------------------------------------------------

@pytest.mark.parametrize("R", [3, 5, 7])
def test_independent_jobs_tac_is_johnson_optimal(R):
    """recv i -> private op i is the two-machine flow shop (channel, then device), for
    which ordering by the pairwise rule of Case 1 is makespan-optimal (Johnson 1954).
    So TAC must reach the brute-force minimum over all R! orders."""
    d = wl.independent_jobs_dag(R)
    dep = deps(d)
    perms = all_orders(R)
    rng = np.random.default_rng(R)
    n_printed_worse = 0
    for trial in range(12):
        rv1, op1 = rand_times(rng, 1, R, 1, 40), rand_times(rng, 1, R, 1, 40)
        rv, op = np.repeat(rv1, len(perms), axis=0), np.repeat(op1, len(perms), axis=0)
        m = sim(d, perms, op, rv)[0]
        order = oracle.tac(dep, d.recv_ids, op1, rv1)[0][0]
        assert sorted(order) == list(range(R))
        m_tac = sim(d, order, op1, rv1)[0][0]
        assert m_tac == m.min()
        printed = oracle.tac(dep, d.recv_ids, op1, rv1, comparator_mode=1)[0][0]
        n_printed_worse += sim(d, printed, op1, rv1)[0][0] > m.min()
    assert n_printed_worse > 0


@pytest.mark.parametrize("seed,R", [(0, 4), (1, 6), (2, 7), (3, 8)])
def test_brute_force_no_order_beats_the_bounds(seed, R):
    d = wl.layered_dag(seed, levels=5, width=4, fan_in=(1, 2), back=2, n_recv=R, attach=(1, 2))
    dep = deps(d)
    depb = dep_bool(dep, R)
    perms = all_orders(R)
    rng = np.random.default_rng(seed)
    rv1, op1 = rand_times(rng, 1, R), rand_times(rng, 1, d.n_compute)
    rv, op = np.repeat(rv1, len(perms), axis=0), np.repeat(op1, len(perms), axis=0)
    m, e, U, L, S = sim(d, perms, op, rv)
    assert (m >= L).all() and (m <= U).all() and (e >= 0).all() and (e <= 1).all()
    np.testing.assert_array_equal(m, closed_form_makespan(depb, d, perms, op, rv))
    best = m.min()
    tac_order = oracle.tac(dep, d.recv_ids, op1, rv1)[0][0]
    tic_order = oracle.tic(dep, d.recv_ids)[1]
    assert sorted(tac_order) == list(range(R)) and sorted(tic_order) == list(range(R))
    assert sim(d, tac_order, op1, rv1)[0][0] >= best
    assert sim(d, tic_order, op1, rv1)[0][0] >= best
    assert best >= L[0]


# --------------------------------------------------------------------------
# invariances
# --------------------------------------------------------------------------

def test_power_of_two_scaling_and_relabelling():
    d = wl.layered_dag(9, levels=6, width=5, fan_in=(1, 3), back=2, n_recv=10, attach=(1, 3))
    dep = deps(d)
    rng = np.random.default_rng(4)
    B = 16
    rv, op = rand_times(rng, B, d.n_recv), rand_times(rng, B, d.n_compute)
    o1, r1, p1, mp1 = oracle.tac(dep, d.recv_ids, op, rv)
    o2, r2, p2, mp2 = oracle.tac(dep, d.recv_ids, op * 8, rv * 8)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(p1 * 8, p2)
    np.testing.assert_array_equal(mp1 * 8, mp2)
    m1, e1, U1, L1, S1 = sim(d, o1, op, rv)
    m2, e2, U2, L2, S2 = sim(d, o1, op * 8, rv * 8)
    np.testing.assert_array_equal(m1 * 8, m2)
    np.testing.assert_array_equal(e1, e2)
    np.testing.assert_array_equal(S1, S2)
    # op ids permuted, recv indices kept: identical orders and makespans
    d2, new_id = wl.relabel(d, 1)
    cmap = wl.compute_column_map(d, d2, new_id)
    dep2 = deps(d2)
    o3 = oracle.tac(dep2, d2.recv_ids, op[:, cmap], rv)[0]
    np.testing.assert_array_equal(o3, o1)
    m3 = sim(d2, o3, op[:, cmap], rv)[0]
    np.testing.assert_array_equal(m3, m1)
    np.testing.assert_array_equal(oracle.tic(dep2, d2.recv_ids)[0], oracle.tic(dep, d.recv_ids)[0])


def test_summation_order_does_not_matter_on_quantised_presets():
    """Times of the presets are multiples of 2**-30 s, so every sum is exact: recv
    indices can be visited in any order without changing a single bit of the result."""
    d = wl.tiny_dag()
    dep = deps(d)
    op, rv = wl.timing_samples(d, 0, 8)
    assert (op == np.rint(op / wl.QUANTUM) * wl.QUANTUM).all() and (op >= wl.QUANTUM).all()
    t = full_time_row(d, op[0], rv[0])
    alive = np.ones(d.n_recv, dtype=np.uint8)
    M, P, Mplus = oracle.update_properties(dep, d.recv_ids, t, alive)
    depb = dep_bool(dep, d.n_recv)
    perm = np.random.default_rng(0).permutation(d.n_recv)
    M_shuffled = np.array([sum(rv[0][i] for i in perm if depb[v, i]) for v in range(d.n_ops)])
    np.testing.assert_array_equal(M, M_shuffled)


def test_partial_rounds_prefix():
    d = wl.tiny_dag()
    dep = deps(d)
    op, rv = wl.timing_samples(d, 0, 4)
    full = oracle.tac(dep, d.recv_ids, op, rv)[0]
    part = oracle.tac(dep, d.recv_ids, op, rv, max_rounds=5)[0]
    np.testing.assert_array_equal(part[:, :5], full[:, :5])
    assert (part[:, 5:] == -1).all()


def test_start_set_continues_a_prefix():
    """Algorithm 3's loop depends on nothing but the current set R of outstanding recvs, so
    starting from R = (all recvs) minus the first k of an order reproduces the rest of that
    order, round by round, with the same P and M+ values.  On the toy graph of Sec. 2.2 the
    start set {recv2} leaves one round that selects recv2 with P = Time(op2) (op2's only
    outstanding dependency) and no M+."""
    d = wl.toy_dag()
    dep = deps(d)
    g = read_golden("fig1_toy.txt")
    rv, op = g["recv_time"][None, :], g["op_time"][None, :]
    o, r, sP, sM = oracle.tac(dep, d.recv_ids, op, rv, alive0=np.array([[0, 1]], dtype=np.uint8))
    assert list(o[0]) == [1, -1] and list(r[0]) == [-1, 0]
    assert sP[0, 1] == op[0, 1] and np.isinf(sM[0, 1])
    for d in (wl.tiny_dag(), wl.layered_dag(11, levels=9, width=7, fan_in=(1, 3), back=3, n_recv=70, attach=(1, 3)),
              wl.case2_dag()):
        dep = deps(d)
        R = d.n_recv
        op, rv = wl.timing_samples(d, 0, 3)
        full, _, fP, fM = oracle.tac(dep, d.recv_ids, op, rv)
        for k in (0, 1, R // 2, R - 1, R):
            alive0 = np.ones((3, R), dtype=np.uint8)
            for b in range(3):
                alive0[b, full[b, :k]] = 0
            rest, rk, sP, sM = oracle.tac(dep, d.recv_ids, op, rv, alive0=alive0)
            np.testing.assert_array_equal(rest[:, :R - k], full[:, k:])
            assert (rest[:, R - k:] == -1).all()
            for b in range(3):
                sel = full[b, k:]
                np.testing.assert_array_equal(sP[b, sel], fP[b, sel])
                np.testing.assert_array_equal(sM[b, sel], fM[b, sel])
                np.testing.assert_array_equal(rk[b, sel], np.arange(R - k))
            one = oracle.tac(dep, d.recv_ids, op, rv, alive0=alive0, max_rounds=1)[0]
            if k < R:
                np.testing.assert_array_equal(one[:, 0], full[:, k])


# --------------------------------------------------------------------------
# Straggler effect (Sec. 6): longest wait over iteration time, per group of workers
# --------------------------------------------------------------------------

def test_straggler_effect_closed_forms():
    # hand-computed: workers that finish at 8, 10 and 5 s wait 2, 0 and 5 s of a 10 s iteration
    assert np.array_equal(oracle.straggler([8.0, 10.0, 5.0], 3), [0.5])
    # identical workers never wait; a single worker has nobody to wait for
    assert np.array_equal(oracle.straggler([3.0, 3.0, 3.0, 3.0], 2), [0.0, 0.0])
    assert np.array_equal(oracle.straggler([1.0, 7.0, 2.0], 1), [0.0, 0.0, 0.0])
    # a worker with nothing to do waits for the whole iteration; an all-zero group gives 0
    assert np.array_equal(oracle.straggler([0.0, 4.0, 0.0, 0.0], 2), [1.0, 0.0])
    # whole groups only: the trailing sample is not used
    assert np.array_equal(oracle.straggler([2.0, 4.0, 100.0], 2), [0.5])
    assert oracle.straggler([], 4).size == 0
    rng = np.random.default_rng(5)
    m = rng.integers(1, 1000, size=96).astype(np.float64)
    for w in (2, 3, 8, 32):
        s = oracle.straggler(m, w)
        g = m[:96 // w * w].reshape(-1, w)
        assert np.array_equal(s, (g.max(axis=1) - g.min(axis=1)) / g.max(axis=1))
        assert np.array_equal(oracle.straggler(m * 8, w), s)                 # scale-free
        assert np.array_equal(oracle.straggler(g[:, ::-1].ravel(), w), s)    # order of the workers
        assert (s >= 0).all() and (s < 1).all()


def test_straggler_effect_of_the_toy_graph_orders():
    """Two workers on the toy graph of Sec. 2.2, one with the good transfer order and one with
    the bad one: the makespans the fixture gives by hand (8 s and 10 s) mean the first worker
    waits 2 s of a 10 s iteration."""
    g = read_golden("fig1_toy.txt")
    d = wl.toy_dag()
    op = np.tile(np.array(g["op_time"], dtype=np.float64), (2, 1))
    rv = np.tile(np.array(g["recv_time"], dtype=np.float64), (2, 1))
    orders = np.array([[0, 1], [1, 0]], dtype=np.int32)
    m = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, orders, op, rv)[0]
    assert m.tolist() == [g["makespan_order_0_1"][0], g["makespan_order_1_0"][0]]
    assert oracle.straggler(m, 2).tolist() == [0.2]
    # both workers on the same order: no straggler, whatever the order
    for o in orders:
        m1 = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, np.tile(o, (2, 1)), op, rv)[0]
        assert oracle.straggler(m1, 2).tolist() == [0.0]


# --------------------------------------------------------------------------
# Several channels (Sec. 4.1, 5.1)
# --------------------------------------------------------------------------

def release_date_makespan(dep_b, chan, n_channels, order, op, rv):
    """The makespan from first principles, for one sample: the channels never wait (recvs are
    roots), so recv r arrives at the sum of the transfer times queued before and including it on its
    channel; a compute op is released when the last recv it depends on has arrived; a device that
    never idles while an op is ready finishes at  max over release dates rho of
    (rho + total time of the ops released at rho or later); the last arrival also bounds it."""
    R = order.size
    arrival = np.zeros(R)
    for c in range(n_channels):
        q = [r for r in order if chan[r] == c]
        arrival[q] = np.cumsum(rv[q])
    rho = (dep_b * arrival[None, :]).max(axis=1) if R else np.zeros(dep_b.shape[0])
    m = arrival.max() if R else 0.0
    for x in np.unique(rho):
        m = max(m, x + op[rho >= x].sum())
    return m


@pytest.mark.parametrize("seed", range(6))
def test_channels_equal_release_date_form_and_reduce_to_one_channel(seed):
    rng = np.random.default_rng(100 + seed)
    R = int(rng.integers(2, 14))
    d = wl.layered_dag(200 + seed, levels=int(rng.integers(2, 6)), width=int(rng.integers(2, 6)), fan_in=(1, 3),
                       back=2, n_recv=R, attach=(1, 3))
    dep = oracle.find_dependencies(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    dep_b = dep_bool(dep, R)[d.compute_ids()]
    B = 12
    op = rng.integers(0, 40, size=(B, d.n_compute)).astype(np.float64) * 0.125
    rv = rng.integers(1, 40, size=(B, R)).astype(np.float64) * 0.125
    orders = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    one = oracle.simulate(*args, orders, op, rv)
    got1 = oracle.simulate_channels(*args, 1, np.zeros(R, np.int32), orders, op, rv)
    for a, b in zip(one, got1):
        assert np.array_equal(a, b)
    prev = one[0]
    for C in (2, 3, R):
        chan = (np.arange(R) % C).astype(np.int32) if C == R else rng.integers(0, C, size=R).astype(np.int32)
        m, e, U, L, S = oracle.simulate_channels(*args, C, chan, orders, op, rv)
        for b in range(B):
            assert m[b] == release_date_makespan(dep_b, chan, C, orders[b], op[b], rv[b])
            per_chan = max(rv[b][chan == c].sum() for c in range(C))
            assert U[b] == op[b].sum() + rv[b].sum() and L[b] == max(op[b].sum(), per_chan)
            assert L[b] <= m[b] <= U[b]
        # a shared order gives the same as the same order repeated per sample
        ms = oracle.simulate_channels(*args, C, chan, orders[0], op, rv)[0]
        mr = oracle.simulate_channels(*args, C, chan, np.tile(orders[0], (B, 1)), op, rv)[0]
        assert np.array_equal(ms, mr)
        if C == R:
            # a channel per recv: every transfer starts at 0, the order plays no role, and no
            # split of the recvs over fewer channels can be faster
            m2 = oracle.simulate_channels(*args, C, chan, orders[:, ::-1].copy(), op, rv)[0]
            assert np.array_equal(m, m2)
            assert (m <= prev).all() and (m <= one[0]).all()
        prev = np.minimum(prev, m) if C != R else prev


def test_channels_toy_graph_by_hand():
    g = read_golden("toy_two_channels.txt")
    d = wl.toy_dag()
    op = np.array([g["op_time"]], dtype=np.float64)
    rv = np.array([g["recv_time"]], dtype=np.float64)
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    for order in ([0, 1], [1, 0]):
        m, e, U, L, S = oracle.simulate_channels(*args, 2, [0, 1], np.array(order, np.int32), op, rv)
        assert (m[0], U[0], L[0]) == (g["makespan_two_channels"][0], g["U"][0], g["L_two_channels"][0])
        assert e[0] == g["E_two_channels"][0] and S[0] == g["S_two_channels"][0]
        m, e, U, L, S = oracle.simulate_channels(*args, 1, [0, 0], np.array(order, np.int32), op, rv)
        key = f"order_{order[0]}_{order[1]}"
        assert m[0] == g["makespan_one_channel_" + key][0] and e[0] == g["E_one_channel_" + key][0]
        assert L[0] == g["L_one_channel"][0] and S[0] == g["S_one_channel"][0]
    # both recvs on channel 1 of two: channel 0 stays empty and nothing changes against one channel
    m = oracle.simulate_channels(*args, 2, [1, 1], np.array([0, 1], np.int32), op, rv)[0]
    assert m[0] == g["makespan_one_channel_order_0_1"][0]


# --------------------------------------------------------------------------
# Time oracle estimator (Sec. 5): minimum over the measured runs
# --------------------------------------------------------------------------

def test_time_oracle_is_the_minimum_of_the_runs():
    # five runs of three ops, by hand
    runs = np.array([[3.0, 9.0, 1.5], [2.5, 9.5, 1.5], [4.0, 8.0, 2.0], [2.75, 8.25, 1.75], [3.5, 9.0, 1.25]])
    assert oracle.time_oracle_min(runs).tolist() == [2.5, 8.0, 1.25]
    assert np.array_equal(oracle.time_oracle_min(runs[:1]), runs[0])                 # one run: itself
    assert np.array_equal(oracle.time_oracle_min(runs[::-1].copy()), [2.5, 8.0, 1.25])  # run order plays no role
    rng = np.random.default_rng(2)
    big = rng.integers(1, 10**6, size=(5, 1000)).astype(np.float64)
    t = oracle.time_oracle_min(big)
    assert np.array_equal(t, np.sort(big, axis=0)[0])
    assert (t[None, :] <= big).all() and (t[None, :] == big).any(axis=0).all()
    # a run that is slower everywhere changes nothing; one that is faster everywhere replaces all
    assert np.array_equal(oracle.time_oracle_min(np.vstack([big, big.max(axis=0) + 1])), t)
    assert np.array_equal(oracle.time_oracle_min(np.vstack([big, t - 1])), t - 1)
    assert oracle.time_oracle_min(np.zeros((5, 0))).size == 0



# --------------------------------------------------------------------------
# order search (Sec. 3.1: the best order is NP-hard to find; Sec. 4.3: the comparator is an
# approximation): a climb through proposed exchanges, measured by the simulated iteration
# --------------------------------------------------------------------------

def search(d, order, moves, op, rv):
    return oracle.order_search(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, order, moves, op, rv)


def test_order_search_toy_graph_and_flow_shop_by_hand():
    g = read_golden("fig1_toy.txt")
    d = wl.toy_dag()
    rv, op = g["recv_time"][None, :], g["op_time"][None, :]
    best, m, m0, acc = search(d, np.array([1, 0]), [[0, 1]], op, rv)          # the bad order is repaired
    assert list(best[0]) == [0, 1] and m[0] == g["makespan_order_0_1"][0] and m0[0] == g["makespan_order_1_0"][0]
    assert acc[0] == 1
    best, m, m0, acc = search(d, np.array([0, 1]), [[0, 1], [1, 0]], op, rv)  # the good one is kept
    assert list(best[0]) == [0, 1] and m[0] == m0[0] == g["makespan_order_0_1"][0] and acc[0] == 0

    f = read_golden("flow_shop_climb.txt")
    d = wl.independent_jobs_dag(3)
    rv, op = f["recv_time"][None, :], f["op_time"][None, :]
    best, m, m0, acc = search(d, f["start_order"].astype(np.int32), f["moves"].astype(np.int32).reshape(-1, 2), op, rv)
    np.testing.assert_array_equal(best[0], f["best_order"].astype(int))
    assert m[0] == f["best_makespan"][0] and m0[0] == f["start_makespan"][0] and acc[0] == f["n_accepted"][0]
    # no moves: the start order comes back
    best, m, m0, acc = search(d, f["start_order"].astype(np.int32), np.zeros((0, 2), dtype=np.int32), op, rv)
    assert list(best[0]) == [0, 1, 2] and m[0] == m0[0] == f["start_makespan"][0] and acc[0] == 0


@pytest.mark.parametrize("seed,R", [(0, 4), (1, 5), (2, 6)])
def test_order_search_ends_where_no_exchange_helps(seed, R):
    """Enough passes over all pairs end in an order that no single exchange improves; every
    figure is re-derived from the closed form of the makespan, which shares nothing with the
    event-driven iteration the search measures with."""
    d = wl.layered_dag(seed, levels=5, width=4, fan_in=(1, 2), back=2, n_recv=R, attach=(1, 2))
    depb = dep_bool(deps(d), R)
    rng = np.random.default_rng(100 + seed)
    B = 6
    rv, op = rand_times(rng, B, R), rand_times(rng, B, d.n_compute)
    start = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)
    pairs = [(a, b) for a in range(R) for b in range(a + 1, R)]
    moves = np.array(pairs * 12, dtype=np.int32)
    best, m, m0, acc = search(d, start, moves, op, rv)
    assert all(sorted(o) == list(range(R)) for o in best)
    np.testing.assert_array_equal(m0, closed_form_makespan(depb, d, start, op, rv))
    np.testing.assert_array_equal(m, closed_form_makespan(depb, d, best, op, rv))
    assert (m <= m0).all() and ((acc > 0) == (m < m0)).all()
    perms = all_orders(R)
    for b in range(B):
        for (pa, pb) in pairs:                       # no exchange improves the end order
            o = best[b].copy()
            o[pa], o[pb] = o[pb], o[pa]
            assert closed_form_makespan(depb, d, o, op[b:b + 1], rv[b:b + 1])[0] >= m[b]
        rvp, opp = np.repeat(rv[b:b + 1], len(perms), axis=0), np.repeat(op[b:b + 1], len(perms), axis=0)
        assert m[b] >= closed_form_makespan(depb, d, perms, opp, rvp).min()     # and none beats brute force
    # the same climb replayed with the closed form as the measure takes the same decisions
    for b in range(B):
        cur = start[b].copy()
        mc = closed_form_makespan(depb, d, cur, op[b:b + 1], rv[b:b + 1])[0]
        n_acc = 0
        for (pa, pb) in moves:
            cur[pa], cur[pb] = cur[pb], cur[pa]
            mm = closed_form_makespan(depb, d, cur, op[b:b + 1], rv[b:b + 1])[0]
            if mm < mc:
                mc, n_acc = mm, n_acc + 1
            else:
                cur[pa], cur[pb] = cur[pb], cur[pa]
        np.testing.assert_array_equal(cur, best[b])
        assert n_acc == acc[b] and mc == m[b]


def test_order_search_shared_start_order():
    d = wl.layered_dag(5, levels=4, width=3, fan_in=(1, 2), back=2, n_recv=5, attach=(1, 2))
    rng = np.random.default_rng(9)
    rv, op = rand_times(rng, 4, 5), rand_times(rng, 4, d.n_compute)
    start = np.array([4, 3, 2, 1, 0], dtype=np.int32)
    moves = rng.integers(0, 5, size=(40, 2)).astype(np.int32)
    a = search(d, start, moves, op, rv)
    b = search(d, np.repeat(start[None, :], 4, axis=0), moves, op, rv)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_near_tie_checker_accepts_the_oracle_and_rejects_a_swap():
    """The checker that the GPU tests use on unquantised times: the oracle's own order passes with no near
    tie; the same order with two steps exchanged is refused unless the round really is a tie."""
    from helpers import tac_order_up_to_near_ties
    d = wl.layered_dag(11, levels=9, width=7, fan_in=(1, 3), back=3, n_recv=70, attach=(1, 3))
    dep = oracle.find_dependencies(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    rng = np.random.default_rng(5)
    op = rng.lognormal(np.log(1e-3), 0.5, size=(4, d.n_compute))
    rv = rng.lognormal(np.log(2e-3), 0.7, size=(4, d.n_recv))
    eo = oracle.tac(dep, d.recv_ids, op, rv)[0]
    refused = 0
    for b in range(4):
        assert tac_order_up_to_near_ties(oracle, d, dep, op[b], rv[b], eo[b]) == 0
        bad = eo[b].copy()
        bad[[3, 4]] = bad[[4, 3]]
        try:
            tac_order_up_to_near_ties(oracle, d, dep, op[b], rv[b], bad)
        except AssertionError:
            refused += 1
    assert refused == 4


# --------------------------------------------------------------------------
# send ops on an uplink (Sec. 2.2)
# --------------------------------------------------------------------------
def toy_with_sends():
    """recv1 -> op1; op2 <- {op1, recv2}; send1 <- op1; send2 <- op2 (ids 0..5 in that order of kinds)."""
    row_ptr = np.array([0, 0, 0, 1, 3, 4, 5], dtype=np.int32)
    col_idx = np.array([0, 2, 1, 2, 3], dtype=np.int32)
    return (wl.Dag("toy_sends", 6, row_ptr, col_idx, np.array([0, 1], dtype=np.int32), np.ones(4), np.ones(2)),
            np.array([4, 5], dtype=np.int32))


def test_sends_toy_graph_by_hand():
    g = read_golden("toy_sends.txt")
    d, sends = toy_with_sends()
    op, rv = g["op_time"][None], g["recv_time"][None]
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, sends)
    for order, tag in (([0, 1], "order_0_1"), ([1, 0], "order_1_0")):
        m, E, U, L, S = oracle.simulate_sends(*args, np.array(order, dtype=np.int32), op, rv)
        assert m[0] == g["makespan_" + tag][0] and U[0] == g["U"][0] and L[0] == g["L"][0]
        assert E[0] == pytest.approx(g["E_" + tag][0], abs=1e-15) and S[0] == pytest.approx(g["S"][0], abs=1e-15)


def test_sends_without_sends_or_with_sends_of_no_duration_are_the_plain_iteration():
    d = wl.layered_dag(21, levels=6, width=5, fan_in=(1, 3), back=2, n_recv=12, attach=(1, 2))
    rng = np.random.default_rng(8)
    B = 16
    op = rng.integers(1, 50, size=(B, d.n_compute)).astype(np.float64) * wl.QUANTUM
    rv = rng.integers(1, 80, size=(B, d.n_recv)).astype(np.float64) * wl.QUANTUM
    orders = np.stack([rng.permutation(d.n_recv) for _ in range(B)]).astype(np.int32)
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    plain = oracle.simulate(*args, orders, op, rv)
    none = oracle.simulate_sends(*args, np.zeros(0, dtype=np.int32), orders, op, rv)
    for a, b in zip(plain, none):
        assert np.array_equal(a, b)
    # leaves turned into sends that take no time: nothing else moves, and U, L lose nothing
    succ = np.bincount(d.col_idx, minlength=d.n_ops)
    leaves = np.array([v for v in d.compute_ids() if succ[v] == 0], dtype=np.int32)
    assert leaves.size >= 2
    cols = np.searchsorted(d.compute_ids(), leaves)
    op0 = op.copy()
    op0[:, cols] = 0.0
    a = oracle.simulate(*args, orders, op0, rv)
    b = oracle.simulate_sends(*args, leaves, orders, op0, rv)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_sends_chain_is_the_two_machine_flow_shop():
    """recv -> c_1 -> c_2 -> ... -> c_k with a send after every c_i: the compute device and the uplink form
    the textbook two-machine flow shop in the order of the chain, C1_i = C1_{i-1} + a_i (after the recv),
    C2_i = max(C2_{i-1}, C1_i) + s_i."""
    k = 9
    n = 1 + 2 * k
    pred = {}
    for i in range(k):
        pred[1 + i] = [0] if i == 0 else [i]              # c_i = op 1 + i
        pred[1 + k + i] = [1 + i]                          # send_i = op 1 + k + i
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    col = []
    for v in range(n):
        col += pred.get(v, [])
        row_ptr[v + 1] = len(col)
    d = wl.Dag("chain_sends", n, row_ptr, np.array(col, dtype=np.int32), np.array([0], dtype=np.int32),
               np.ones(2 * k), np.ones(1))
    sends = np.arange(1 + k, n, dtype=np.int32)
    rng = np.random.default_rng(9)
    B = 32
    op = rng.lognormal(0.0, 0.8, size=(B, 2 * k))
    rv = rng.lognormal(0.0, 0.5, size=(B, 1))
    m = oracle.simulate_sends(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, sends, np.zeros(1, dtype=np.int32), op, rv)[0]
    for b in range(B):
        c1, c2 = rv[b, 0], 0.0
        for i in range(k):
            c1 = c1 + op[b, i]
            c2 = max(c2, c1) + op[b, k + i]
        assert m[b] == pytest.approx(max(c1, c2), rel=1e-14)


@pytest.mark.parametrize("seed", range(12))
def test_sends_equal_a_tick_by_tick_simulation(seed):
    from helpers import tick_simulate_sends
    rng = np.random.default_rng(100 + seed)
    d = wl.layered_dag(300 + seed, levels=int(rng.integers(2, 5)), width=int(rng.integers(2, 5)), fan_in=(1, 3),
                       back=2, n_recv=int(rng.integers(1, 6)), attach=(1, 2))
    succ = np.bincount(d.col_idx, minlength=d.n_ops)
    leaves = [int(v) for v in d.compute_ids() if succ[v] == 0]
    sends = np.array([v for v in leaves if rng.random() < 0.7] or leaves[:1], dtype=np.int32)
    B = 6
    op = rng.integers(0, 6, size=(B, d.n_compute)).astype(np.float64)       # zeros included
    rv = rng.integers(0, 7, size=(B, d.n_recv)).astype(np.float64)
    orders = np.stack([rng.permutation(d.n_recv) for _ in range(B)]).astype(np.int32)
    m = oracle.simulate_sends(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, sends, orders, op, rv)[0]
    for b in range(B):
        assert m[b] == tick_simulate_sends(d, sends, orders[b], op[b], rv[b]), (seed, b)


def test_sends_the_pick_of_the_compute_device_matters():
    """Without sends the makespan does not depend on which ready op the device takes; with sends it does,
    which is why the pick is part of the reading: two ready ops, the one with the long send behind it should
    go first."""
    # recv0 -> a (op 1), recv0 -> b (op 2); send after a (op 3, long), send after b (op 4, short)
    row_ptr = np.array([0, 0, 1, 2, 3, 4], dtype=np.int32)
    col_idx = np.array([0, 0, 1, 2], dtype=np.int32)
    args = (5, row_ptr, col_idx, np.array([0], dtype=np.int32), np.array([3, 4], dtype=np.int32), np.zeros(1, dtype=np.int32))
    op = np.array([[2.0, 2.0, 10.0, 1.0]])
    rv = np.array([[1.0]])
    low = oracle.simulate_sends(*args, op, rv)[0][0]                                      # a first: 1..3, send 3..13; b 3..5, send 13..14
    high = oracle.simulate_sends(*args, op, rv, pick_key=np.array([0, 2, 1, 0, 0]))[0][0]   # b first: 1..3, send 3..4; a 3..5, send 5..15
    assert low == 14.0 and high == 15.0
