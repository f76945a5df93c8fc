"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer outputs (bitsets, TIC priorities, orders, ranks) must be
bit-exact; float64 outputs within 1e-5 relative (they are in fact exact on the presets,
whose times are multiples of 2**-30 s)."""

import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle
from paper_1803_03288_amd import workloads as wl

from helpers import dep_bool, oracle_rounds_after_prefix, oracle_tac_rows, tac_order_up_to_near_ties

RTOL = 1e-5


@pytest.fixture(scope="module")
def tt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1803_03288_amd import binding
    binding.lib()            # raises if the library has not been built
    return binding


_cache = {}


def get(tt, name, maker=None):
    """(Dag description, GPU handle, oracle dep matrix), cached per name."""
    if name not in _cache:
        d = maker() if maker else wl.preset(name)
        print(f"[build] {name}: n={d.n_ops} R={d.n_recv} E={d.n_edges}", flush=True)
        h = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
        dep = oracle.find_dependencies(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
        _cache[name] = (d, h, dep)
    return _cache[name]


def cuda(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def subset_rows(B, k):
    """first k/2 samples + k/2 strided over the batch"""
    k = min(k, B)
    first = list(range(k // 2))
    rest = sorted(set(np.linspace(k // 2, B - 1, k - k // 2).astype(int).tolist()) - set(first))
    return first + rest


SMALL = {
    "layered70": lambda: wl.layered_dag(11, levels=9, width=7, fan_in=(1, 3), back=3, n_recv=70, attach=(1, 3)),
    "relabel": lambda: wl.relabel(wl.layered_dag(12, levels=8, width=6, fan_in=(1, 3), back=2, n_recv=40,
                                                 attach=(1, 4)), 5)[0],
    "chain": lambda: wl.chain_dag(33),
    # the largest graph the wave-per-sample kernels take: 512 recvs, 512 classes (eight per lane)
    "chain512": lambda: wl.chain_dag(512, name="chain512"),
    "jobs": lambda: wl.independent_jobs_dag(9),
    "funnel": lambda: wl.funnel_dag(6, 9),
    "toy": wl.toy_dag,
    "case2": wl.case2_dag,
    "single": lambda: wl.chain_dag(1),
    "mini_stress": lambda: wl.stress_dag(levels=40, width=50, n_recv=300, seed=14, batch=64),
    # a level wider than one pass of the propagation workgroup (W = 18 words, 1 500 ops per level)
    "wide_levels": lambda: wl.layered_dag(21, levels=4, width=1500, fan_in=(2, 3), back=1, n_recv=1100, attach=(1, 3)),
    # deep and narrow with edges that span thousands of positions: inputs that have left the LDS ring
    "long_edges": lambda: wl.deep_narrow_dag(22, levels=2500, width=4, n_recv=60),
    # the same with wider rows (W = 3 words, four-word slices; W = 2 words, two-word slices)
    "long_edges_w3": lambda: wl.deep_narrow_dag(23, levels=1300, width=4, n_recv=150),
    "long_edges_w2": lambda: wl.deep_narrow_dag(27, levels=1500, width=4, n_recv=100),
    # narrow levels and many words per row (one wave per one-word slice, eighteen slices)
    "narrow_w18": lambda: wl.deep_narrow_dag(29, levels=300, width=4, n_recv=1100),
    # two-word rows with a level wider than one pass of the propagation workgroup
    "wide_levels_w2": lambda: wl.layered_dag(28, levels=4, width=700, fan_in=(2, 3), back=1, n_recv=100, attach=(1, 3)),
    # levels of a hundred ops (several waves per workgroup: the level-major kernel) with edges that reach
    # back past the rows kept in LDS, for one-, two- and four-word slices
    "deep_w1": lambda: wl.deep_narrow_dag(24, levels=700, width=100, n_recv=60),
    "deep_w2": lambda: wl.deep_narrow_dag(25, levels=400, width=70, n_recv=100),
    "deep_w3": lambda: wl.deep_narrow_dag(26, levels=500, width=40, n_recv=150),
}
PRESETS = ["tiny", "resnet50", "vgg16", "inception3", "stress"]


# --------------------------------------------------------------------------
# dependency bitsets and TIC: bit-exact on every preset at full size
# --------------------------------------------------------------------------

@pytest.mark.parametrize("name", PRESETS + list(SMALL))
def test_deps_and_tic_bit_exact(tt, name):
    d, h, dep = get(tt, name, SMALL.get(name))
    assert (h.n_ops, h.n_recv, h.words) == (d.n_ops, d.n_recv, d.words)
    got = h.deps().cpu().numpy().view(np.uint64)
    assert got.shape == dep.shape
    assert np.array_equal(got, dep)
    prio, order, rank = (x.cpu().numpy() for x in tt.tic_priority(h))
    eprio, eorder, erank = oracle.tic(dep, d.recv_ids)
    assert np.array_equal(prio, eprio)
    assert np.array_equal(order, eorder)
    assert np.array_equal(rank, erank)
    # number of classes reported = number of distinct non-empty rows among compute ops
    rows = dep[d.compute_ids()]
    assert h.n_classes == np.unique(rows, axis=0).shape[0]


@pytest.mark.parametrize("name", ["stress", "deep_w1", "deep_w2", "deep_w3", "resnet50", "tiny"])
def test_deps_of_several_handles_in_one_launch(tt, name):
    """tictac_dag_recompute_deps_batch: the bitsets of several handles, cleared first, are propagated again by
    one call (one launch where the graphs take the level-major kernel, one after the other elsewhere) and
    equal the oracle's; so do those of the single-handle call."""
    d, h, dep = get(tt, name, SMALL.get(name))
    hs = [tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids) for _ in range(3)]
    for x in hs:
        x.deps_view().zero_()
    tt.recompute_deps_batch(hs)
    for x in hs:
        assert np.array_equal(x.deps().cpu().numpy().view(np.uint64), dep)
    hs[1].deps_view().fill_(-1)
    hs[1].recompute_deps()
    assert np.array_equal(hs[1].deps().cpu().numpy().view(np.uint64), dep)
    tt.recompute_deps_batch(hs[:1])
    tt.recompute_deps_batch([])
    assert np.array_equal(hs[0].deps().cpu().numpy().view(np.uint64), dep)
    for x in hs:
        x.close()


def test_deps_of_different_graphs_in_one_call(tt):
    """tictac_dag_recompute_deps_batch on handles of different graphs: graphs of one size and one launch shape share
    a launch (the kernel with 64-byte slices here: rows of 16 words), a graph of another size in the same list
    sends the call through one launch per handle; either way every handle gets its own bitsets."""
    graphs = [wl.stress_dag(levels=40, width=120, n_recv=1024, seed=s, batch=4) for s in (61, 62, 63)]
    graphs.append(wl.stress_dag(levels=25, width=90, n_recv=512, seed=64, batch=4))
    deps = [oracle.find_dependencies(g.n_ops, g.row_ptr, g.col_idx, g.recv_ids) for g in graphs]
    hs = [tt.build_deps(g.n_ops, g.row_ptr, g.col_idx, g.recv_ids) for g in graphs]
    for group in (hs[:3], hs, [hs[3], hs[0]]):
        for x in group:
            x.deps_view().zero_()
        tt.recompute_deps_batch(group)
        for x in group:
            i = hs.index(x)
            assert np.array_equal(x.deps().cpu().numpy().view(np.uint64), deps[i]), i
    for x in hs:
        x.close()


def test_no_recvs_and_empty_graph(tt):
    d = wl.no_recv_dag(17)
    h = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    assert h.words == 0 and h.deps().numel() == 0
    prio, order, rank = tt.tic_priority(h)
    assert prio.numel() == 0
    rng = np.random.default_rng(0)
    op = rng.integers(1, 100, size=(5, 17)).astype(np.float64) * wl.QUANTUM
    rv = np.zeros((5, 0))
    o = tt.tac_priority(h, cuda(op), cuda(rv))[0]
    assert tuple(o.shape) == (5, 0)
    m, e, U, L, S = (x.cpu().numpy() for x in tt.simulate(h, torch.zeros(0, dtype=torch.int32, device="cuda"),
                                                          cuda(op), cuda(rv)))
    em, ee, eU, eL, eS = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, np.zeros(0, np.int32), op, rv)
    for a, b in ((m, em), (e, ee), (U, eU), (L, eL), (S, eS)):
        assert np.array_equal(a, b)
    res = tt.tac_simulate(h, cuda(op), cuda(rv))
    assert np.array_equal(res[4].cpu().numpy(), em) and np.array_equal(res[5].cpu().numpy(), ee)
    # empty graph and B = 0
    h0 = tt.build_deps(0, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32))
    assert h0.n_ops == 0
    d1, h1, _ = get(tt, "toy", wl.toy_dag)
    o = tt.tac_priority(h1, torch.zeros((0, 2), dtype=torch.float64, device="cuda"),
                        torch.zeros((0, 2), dtype=torch.float64, device="cuda"))[0]
    assert tuple(o.shape) == (0, 2)


# --------------------------------------------------------------------------
# TAC and simulation
# --------------------------------------------------------------------------

def run_tac_sim_parity(tt, d, h, dep, op, rv, tag):
    """TAC (order, rank, sel_P, sel_Mplus), simulation under the TAC order (per-sample
    orders), the fused call, and simulation under the shared TIC order: all against the
    oracle, element by element."""
    print(f"[parity] {tag}: B={op.shape[0]}", flush=True)
    R = d.n_recv
    eo, er, eP, eM = oracle.tac(dep, d.recv_ids, op, rv)
    gop, grv = cuda(op), cuda(rv)
    o, r, sP, sM = tt.tac_priority(h, gop, grv, want_rank=True, want_sel=True)
    o, r, sP, sM = o.cpu().numpy(), r.cpu().numpy(), sP.cpu().numpy(), sM.cpu().numpy()
    assert np.array_equal(o, eo), f"{tag}: TAC order differs in {(o != eo).any(axis=1).sum()} samples"
    assert np.array_equal(r, er)
    np.testing.assert_allclose(sP, eP, rtol=RTOL, atol=0)
    assert np.array_equal(np.isinf(sM), np.isinf(eM))
    fin = np.isfinite(eM)
    np.testing.assert_allclose(sM[fin], eM[fin], rtol=RTOL, atol=0)

    exp = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, eo, op, rv)
    got = [x.cpu().numpy() for x in tt.simulate(h, cuda(eo), gop, grv)]
    for a, b, nm in zip(got, exp, "m E U L S".split()):
        np.testing.assert_allclose(a, b, rtol=RTOL, atol=1e-300, err_msg=f"{tag}: simulate {nm}")
    fused = tt.tac_simulate(h, gop, grv, want_rank=True, want_sel=True)
    assert np.array_equal(fused[0].cpu().numpy(), eo)
    assert np.array_equal(fused[1].cpu().numpy(), er)
    for a, b, nm in zip(fused[4:], exp, "m E U L S".split()):
        np.testing.assert_allclose(a.cpu().numpy(), b, rtol=RTOL, atol=1e-300, err_msg=f"{tag}: fused {nm}")
    # the presets are quantised: results are exact, not merely close
    assert np.array_equal(got[0], exp[0]) and np.array_equal(fused[4].cpu().numpy(), exp[0])
    # the same two calls without the per-round outputs: small graphs then run in the
    # one-wave-per-sample kernels that the benchmark times
    o2, r2 = tt.tac_priority(h, gop, grv, want_rank=True)[:2]
    assert np.array_equal(o2.cpu().numpy(), eo), f"{tag}: TAC order (no sel) differs"
    assert np.array_equal(r2.cpu().numpy(), er)
    fused2 = tt.tac_simulate(h, gop, grv, want_rank=True)
    assert np.array_equal(fused2[0].cpu().numpy(), eo), f"{tag}: fused order (no sel) differs"
    assert np.array_equal(fused2[1].cpu().numpy(), er)
    for a, b, nm in zip(fused2[4:], exp, "m E U L S".split()):
        np.testing.assert_allclose(a.cpu().numpy(), b, rtol=RTOL, atol=1e-300, err_msg=f"{tag}: fused (no sel) {nm}")
    assert np.array_equal(fused2[4].cpu().numpy(), exp[0])
    o3 = tt.tac_priority(h, gop, grv)[0]
    assert np.array_equal(o3.cpu().numpy(), eo)

    if R:
        tic_order = oracle.tic(dep, d.recv_ids)[1]
        exp2 = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, tic_order, op, rv)
        got2 = [x.cpu().numpy() for x in tt.simulate(h, cuda(tic_order), gop, grv)]
        for a, b, nm in zip(got2, exp2, "m E U L S".split()):
            np.testing.assert_allclose(a, b, rtol=RTOL, atol=1e-300, err_msg=f"{tag}: simulate(TIC) {nm}")
    return o


@pytest.mark.parametrize("name,k", [("tiny", 1024), ("vgg16", 1024), ("resnet50", 96), ("inception3", 6)])
def test_tac_and_simulate_presets(tt, name, k):
    d, h, dep = get(tt, name)
    rows = subset_rows(d.batch, k)
    op, rv = wl.sample_rows(d, rows)
    run_tac_sim_parity(tt, d, h, dep, op, rv, name)


@pytest.mark.parametrize("name", ["layered70", "relabel", "chain", "chain512", "jobs", "funnel", "toy", "case2", "single",
                                  "mini_stress"])
def test_tac_and_simulate_small_graphs(tt, name):
    d, h, dep = get(tt, name, SMALL[name])
    B = 8 if name == "mini_stress" else 200
    op, rv = wl.timing_samples(d, 0, B)
    run_tac_sim_parity(tt, d, h, dep, op, rv, name)


@pytest.mark.parametrize("name", ["layered70", "jobs", "tiny", "case2"])
def test_ties_and_zero_times(tt, name):
    """Times drawn from a handful of values give many exact ties in the comparator; zero
    transfer times force the literal selection path; zero compute times leave P at 0."""
    d, h, dep = get(tt, name, SMALL.get(name))
    rng = np.random.default_rng(3)
    B = 300
    op = rng.integers(0, 4, size=(B, d.n_compute)).astype(np.float64) * 0.25
    rv = rng.integers(1, 4, size=(B, d.n_recv)).astype(np.float64) * 0.25
    run_tac_sim_parity(tt, d, h, dep, op, rv, name + "/ties")
    rv0 = rv.copy()
    rv0[rng.random(rv0.shape) < 0.2] = 0.0
    run_tac_sim_parity(tt, d, h, dep, op, rv0, name + "/zero-transfers")


@pytest.mark.parametrize("n_recv", [63, 64, 65, 128, 129])
def test_word_boundaries_and_ragged_batches(tt, n_recv):
    """Recv counts at and around multiples of the 64-bit word, batches that do not fill a
    workgroup of four waves (1 and 7 samples)."""
    name = f"r{n_recv}"
    d, h, dep = get(tt, name, lambda: wl.layered_dag(30 + n_recv, levels=7, width=9, fan_in=(1, 3), back=2,
                                                      n_recv=n_recv, attach=(1, 3)))
    assert np.array_equal(h.deps().cpu().numpy().view(np.uint64), dep)
    for B in (1, 7):
        op, rv = wl.timing_samples(d, 0, B)
        run_tac_sim_parity(tt, d, h, dep, op, rv, f"{name}/B{B}")


def run_other_calls_parity(tt, d, h, dep, op, rv, rng, tag):
    """Order search, several channels and float32 storage against the oracle on one graph."""
    R, B = d.n_recv, rv.shape[0]
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    gop, grv = cuda(op), cuda(rv)
    orders = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)
    gord = cuda(orders)
    if R <= 512 and h.n_classes <= 512:
        moves = rng.integers(0, R, size=(60, 2)).astype(np.int32)
        exp = oracle.order_search(*args, orders, moves, op, rv)
        got = tt.order_search(h, gord, cuda(moves), gop, grv)
        for a, b, nm in zip(got, exp, ("best_order", "best_makespan", "start_makespan", "n_accepted")):
            assert np.array_equal(a.cpu().numpy(), b), f"{tag}: search {nm}"
        n_ch = int(rng.integers(1, 6))
        chan = rng.integers(0, n_ch, size=R).astype(np.int32)
        exp = oracle.simulate_channels(*args, n_ch, chan, orders, op, rv)
        got = tt.simulate_channels(h, n_ch, chan, gord, gop, grv)
        for a, b, nm in zip(got, exp, "m E U L S".split()):
            assert np.array_equal(a.cpu().numpy(), b), f"{tag}: {n_ch} channels {nm}"
    op32, rv32 = op.astype(np.float32), rv.astype(np.float32)
    op64, rv64 = op32.astype(np.float64), rv32.astype(np.float64)
    eo = oracle.tac(dep, d.recv_ids, op64, rv64)[0]
    exp = oracle.simulate(*args, eo, op64, rv64)
    got = tt.tac_simulate(h, cuda(op32), cuda(rv32))
    assert np.array_equal(got[0].cpu().numpy(), eo), f"{tag}: float32 order"
    for a, b, nm in zip(got[4:], exp, "m E U L S".split()):
        assert np.array_equal(a.cpu().numpy(), b), f"{tag}: float32 fused {nm}"
    exp = oracle.simulate(*args, orders, op64, rv64)
    got = tt.simulate(h, gord, cuda(op32), cuda(rv32))
    for a, b, nm in zip(got, exp, "m E U L S".split()):
        assert np.array_equal(a.cpu().numpy(), b), f"{tag}: float32 simulate {nm}"


@pytest.mark.parametrize("seed", range(int(os.environ.get("TICTAC_TEST_SEEDS", "32"))))
def test_random_graphs(tt, seed):
    """Seeded random layered graphs of varied shape (1 to 200 recvs, shallow and deep, sparse and
    dense attachment), each with ordinary samples and with samples drawn from three values
    (ties everywhere, zero-time ops)."""
    rng = np.random.default_rng(1000 + seed)
    R = int(rng.choice([1, 2, 3, 5, 17, 40, 64, 65, 100, 130, 200]))
    levels, width = int(rng.integers(1, 12)), int(rng.integers(1, 10))
    hi_attach = int(rng.integers(1, 6))
    d = wl.layered_dag(500 + seed, levels=levels, width=width, fan_in=(1, int(rng.integers(1, 4))),
                       back=int(rng.integers(1, 4)), n_recv=R, attach=(1, hi_attach))
    print(f"[random] seed {seed}: R={R} levels={levels} width={width} attach<= {hi_attach}", flush=True)
    h = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    dep = oracle.find_dependencies(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    assert np.array_equal(h.deps().cpu().numpy().view(np.uint64), dep)
    B = 24
    op, rv = wl.timing_samples(d, 0, B)
    run_tac_sim_parity(tt, d, h, dep, op, rv, f"random{seed}")
    op3 = rng.integers(0, 3, size=(B, d.n_compute)).astype(np.float64) * 0.5
    rv3 = rng.integers(1, 3, size=(B, R)).astype(np.float64) * 0.5
    run_tac_sim_parity(tt, d, h, dep, op3, rv3, f"random{seed}/ties")
    run_other_calls_parity(tt, d, h, dep, op, rv, rng, f"random{seed}")
    run_other_calls_parity(tt, d, h, dep, op3, rv3, rng, f"random{seed}/ties")
    h.close()


def test_random_orders_per_sample(tt):
    d, h, dep = get(tt, "layered70", SMALL["layered70"])
    rng = np.random.default_rng(8)
    B = 500
    op, rv = wl.timing_samples(d, 0, B)
    orders = np.stack([rng.permutation(d.n_recv) for _ in range(B)]).astype(np.int32)
    exp = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, orders, op, rv)
    got = [x.cpu().numpy() for x in tt.simulate(h, cuda(orders), cuda(op), cuda(rv))]
    for a, b in zip(got, exp):
        assert np.array_equal(a, b)


def test_random_order_baseline_and_straggler_effect(tt):
    """The no-scheduling baseline (one random transfer order per sample) against TIC and TAC on the
    same samples, and the straggler effect of groups of w workers: simulation and group
    reduction equal to the oracle, element by element."""
    d, h, dep = get(tt, "resnet50")
    B = 96
    op, rv = wl.timing_samples(d, 0, B)
    orders = wl.random_orders(d, 0, B)
    assert np.array_equal(np.sort(orders, axis=1), np.tile(np.arange(d.n_recv, dtype=np.int32), (B, 1)))
    gop, grv = cuda(op), cuda(rv)
    exp = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, orders, op, rv)
    got = tt.simulate(h, cuda(orders), gop, grv)
    for a, b in zip(got, exp):
        assert np.array_equal(a.cpu().numpy(), b)
    m_tac = tt.tac_simulate(h, gop, grv)[4]
    m_tic = tt.simulate(h, tt.tic_priority(h)[1], gop, grv)[0]
    for m in (got[0], m_tac, m_tic):
        mh = m.cpu().numpy()
        for w in (1, 2, 3, 4, 5, 8, 16, 96, 97):
            s = tt.straggler_effect(m, w).cpu().numpy()
            assert np.array_equal(s, oracle.straggler(mh, w)), w
    # a random order is never better than the lower bound and, here, worse than TAC on average
    assert (got[0].cpu().numpy() >= exp[3]).all()
    assert got[0].mean() > m_tac.mean()
    # degenerate inputs
    assert tt.straggler_effect(torch.zeros(0, dtype=torch.float64, device="cuda"), 4).numel() == 0
    z = tt.straggler_effect(torch.zeros(8, dtype=torch.float64, device="cuda"), 4).cpu().numpy()
    assert np.array_equal(z, [0.0, 0.0])
    big = torch.from_numpy(np.random.default_rng(1).integers(1, 10**6, size=5000).astype(np.float64)).cuda()
    for w in (7, 64, 65, 1000, 5000):
        assert np.array_equal(tt.straggler_effect(big, w).cpu().numpy(), oracle.straggler(big.cpu().numpy(), w))


@pytest.mark.parametrize("name", ["tiny", "layered70", "jobs", "funnel", "toy", "single", "r64", "r129", "chain512",
                                  "resnet50", "inception3"])
def test_several_channels(tt, name):
    """tictac_simulate_channels against the oracle: 1, 2, 3, 4 and 64 channels (and a channel per
    recv where there are at most 64), random and round-robin assignments, per-sample and
    shared orders; one channel equals tictac_simulate."""
    makers = dict(SMALL)
    makers["r64"] = lambda: wl.layered_dag(94, levels=7, width=9, fan_in=(1, 3), back=2, n_recv=64, attach=(1, 3))
    makers["r129"] = lambda: wl.layered_dag(159, levels=7, width=9, fan_in=(1, 3), back=2, n_recv=129, attach=(1, 3))
    d, h, dep = get(tt, name, makers.get(name))
    R = d.n_recv
    B = {"resnet50": 24, "inception3": 4, "chain512": 9}.get(name, 37)
    op, rv = wl.timing_samples(d, 0, B)
    rng = np.random.default_rng(17)
    orders = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)
    gop, grv, gord = cuda(op), cuda(rv), cuda(orders)
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    one = [x.cpu().numpy() for x in tt.simulate(h, gord, gop, grv)]
    got = [x.cpu().numpy() for x in tt.simulate_channels(h, 1, np.zeros(R, np.int32), gord, gop, grv)]
    for a, b in zip(one, got):
        assert np.array_equal(a, b)
    cases = [(2, rng.integers(0, 2, size=R)), (3, np.arange(R) % 3), (4, rng.integers(0, 4, size=R)),
             (64, rng.integers(0, 64, size=R)), (5, np.full(R, 4))]
    if R <= 64:
        cases.append((max(R, 1), np.arange(R)))
    for C, chan in cases:
        chan = chan.astype(np.int32)
        exp = oracle.simulate_channels(*args, C, chan, orders, op, rv)
        got = tt.simulate_channels(h, C, chan, gord, gop, grv)
        for a, b, nm in zip(got, exp, "m E U L S".split()):
            assert np.array_equal(a.cpu().numpy(), b), f"{name}: {C} channels, {nm}"
        exp = oracle.simulate_channels(*args, C, chan, orders[0], op, rv)
        got = tt.simulate_channels(h, C, chan, gord[0].contiguous(), gop, grv)
        for a, b, nm in zip(got, exp, "m E U L S".split()):
            assert np.array_equal(a.cpu().numpy(), b), f"{name}: {C} channels, shared order, {nm}"
    # zero-length transfers and zero-time ops (equal arrivals, equal release dates)
    op0, rv0 = op.copy(), rv.copy()
    op0[rng.random(op0.shape) < 0.3] = 0.0
    rv0[rng.random(rv0.shape) < 0.3] = 0.0
    chan = rng.integers(0, 3, size=R).astype(np.int32)
    exp = oracle.simulate_channels(*args, 3, chan, orders, op0, rv0)
    got = tt.simulate_channels(h, 3, chan, gord, cuda(op0), cuda(rv0))
    for a, b in zip(got, exp):
        assert np.array_equal(a.cpu().numpy(), b)


def test_several_channels_limits(tt):
    from paper_1803_03288_amd.binding import TicTacError
    d, h, dep = get(tt, "toy", wl.toy_dag)
    op, rv = wl.timing_samples(d, 0, 4)
    o = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    for C, chan, code in ((0, [0, 0], -9), (65, [0, 0], -9), (2, [0, 2], -6), (2, [-1, 0], -6)):
        with pytest.raises(TicTacError) as e:
            tt.simulate_channels(h, C, np.array(chan, np.int32), o, cuda(op), cuda(rv))
        assert e.value.code == code
    ds, hs, _ = get(tt, "stress")
    with pytest.raises(TicTacError) as e:
        tt.simulate_channels(hs, 2, np.zeros(ds.n_recv, np.int32), torch.zeros(ds.n_recv, dtype=torch.int32, device="cuda"),
                             torch.zeros((1, ds.n_compute), dtype=torch.float64, device="cuda"),
                             torch.zeros((1, ds.n_recv), dtype=torch.float64, device="cuda"))
    assert e.value.code == -9
    # no recvs: the channels play no role
    dn = wl.no_recv_dag(17)
    hn = tt.build_deps(dn.n_ops, dn.row_ptr, dn.col_idx, dn.recv_ids)
    opn = np.arange(1, 3 * 17 + 1, dtype=np.float64).reshape(3, 17) * wl.QUANTUM
    got = tt.simulate_channels(hn, 3, np.zeros(0, np.int32), torch.zeros(0, dtype=torch.int32, device="cuda"),
                               cuda(opn), cuda(np.zeros((3, 0))))
    assert np.array_equal(got[0].cpu().numpy(), opn.sum(axis=1))


EXTRA = {
    "r64": lambda: wl.layered_dag(94, levels=7, width=9, fan_in=(1, 3), back=2, n_recv=64, attach=(1, 3)),
    "r129": lambda: wl.layered_dag(159, levels=7, width=9, fan_in=(1, 3), back=2, n_recv=129, attach=(1, 3)),
}


@pytest.mark.parametrize("name", ["tiny", "layered70", "jobs", "funnel", "toy", "case2", "single", "chain", "chain512",
                                  "r64", "r129", "resnet50", "vgg16", "inception3"])
def test_order_search(tt, name):
    """tictac_order_search against the oracle: the orders the samples end with, both makespans
    and the number of kept exchanges, from random start orders per sample and from the TIC
    order for all samples; moves include exchanges of a position with itself and positions
    outside the order.  The makespan it reports is the one tictac_simulate gives for that order."""
    makers = dict(SMALL)
    makers.update(EXTRA)
    d, h, dep = get(tt, name, makers.get(name))
    R = d.n_recv
    B, n_moves = {"resnet50": (10, 48), "vgg16": (40, 48), "inception3": (3, 24), "chain512": (9, 80)}.get(name, (37, 150))
    print(f"[order_search] {name}: R={R} B={B} moves={n_moves}", flush=True)
    op, rv = wl.timing_samples(d, 0, B)
    rng = np.random.default_rng(29)
    start = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)
    moves = rng.integers(0, R, size=(n_moves, 2)).astype(np.int32)
    moves[3] = (-1, 0)
    moves[7] = (0, R)
    moves[11] = (R - 1, R - 1)
    gop, grv = cuda(op), cuda(rv)
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    tic_order = oracle.tic(dep, d.recv_ids)[1].astype(np.int32)
    for st in (start, tic_order):
        exp = oracle.order_search(*args, st, moves, op, rv)
        got = tt.order_search(h, cuda(st), cuda(moves), gop, grv)
        for a, b, nm in zip(got, exp, ("best_order", "best_makespan", "start_makespan", "n_accepted")):
            assert np.array_equal(a.cpu().numpy(), b), f"{name}: {nm}"
        again = tt.simulate(h, got[0], gop, grv)[0]
        assert torch.equal(again, got[1])
    # no moves: the start orders come back with their makespans
    got = tt.order_search(h, cuda(start), torch.zeros((0, 2), dtype=torch.int32, device="cuda"), gop, grv)
    assert np.array_equal(got[0].cpu().numpy(), start) and torch.equal(got[1], got[2])
    assert int(got[3].abs().sum()) == 0
    # zero-length transfers and zero-time ops (many equal makespans: nothing is kept on a tie)
    op0, rv0 = op.copy(), rv.copy()
    op0[rng.random(op0.shape) < 0.3] = 0.0
    rv0[rng.random(rv0.shape) < 0.3] = 0.0
    exp = oracle.order_search(*args, start, moves, op0, rv0)
    got = tt.order_search(h, cuda(start), cuda(moves), cuda(op0), cuda(rv0))
    for a, b in zip(got, exp):
        assert np.array_equal(a.cpu().numpy(), b)


def test_order_search_limits(tt):
    from paper_1803_03288_amd.binding import TicTacError
    ds, hs, _ = get(tt, "stress")
    mv = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(TicTacError) as e:
        tt.order_search(hs, torch.zeros(ds.n_recv, dtype=torch.int32, device="cuda"), mv,
                        torch.zeros((1, ds.n_compute), dtype=torch.float64, device="cuda"),
                        torch.zeros((1, ds.n_recv), dtype=torch.float64, device="cuda"))
    assert e.value.code == -9
    # one recv more than the kernel takes; the single-channel simulation still serves such a graph
    d513, h513, _ = get(tt, "chain513", lambda: wl.chain_dag(513, name="chain513"))
    op513, rv513 = wl.timing_samples(d513, 0, 3)
    o513 = torch.arange(513, dtype=torch.int32, device="cuda")
    with pytest.raises(TicTacError) as e:
        tt.order_search(h513, o513, mv, cuda(op513), cuda(rv513))
    assert e.value.code == -9
    with pytest.raises(TicTacError) as e:
        tt.simulate_channels(h513, 2, np.zeros(513, np.int32), o513, cuda(op513), cuda(rv513))
    assert e.value.code == -9
    exp = oracle.simulate(d513.n_ops, d513.row_ptr, d513.col_idx, d513.recv_ids, np.arange(513, dtype=np.int32), op513, rv513)
    got = tt.simulate(h513, o513, cuda(op513), cuda(rv513))
    for a, b in zip(got, exp):
        assert np.array_equal(a.cpu().numpy(), b)
    dn = wl.no_recv_dag(17)
    hn = tt.build_deps(dn.n_ops, dn.row_ptr, dn.col_idx, dn.recv_ids)
    with pytest.raises(TicTacError) as e:
        tt.order_search(hn, torch.zeros(0, dtype=torch.int32, device="cuda"), mv,
                        torch.zeros((2, 17), dtype=torch.float64, device="cuda"),
                        torch.zeros((2, 0), dtype=torch.float64, device="cuda"))
    assert e.value.code == -9
    # an empty batch is valid
    d, h, _ = get(tt, "toy", wl.toy_dag)
    got = tt.order_search(h, torch.tensor([0, 1], dtype=torch.int32, device="cuda"), mv,
                          torch.zeros((0, d.n_compute), dtype=torch.float64, device="cuda"),
                          torch.zeros((0, 2), dtype=torch.float64, device="cuda"))
    assert got[0].shape == (0, 2)


@pytest.mark.parametrize("name,k", [("tiny", 256), ("resnet50", 48), ("vgg16", 512), ("inception3", 4), ("layered70", 64),
                                    ("jobs", 64), ("toy", 16), ("single", 8), ("funnel", 16), ("r129", 32), ("chain512", 6)])
def test_float32_timing_arrays(tt, name, k):
    """tictac_tac_simulate_f32 and tictac_simulate_f32: the timing samples stored as float32.  The
    oracle is given the same rounded values (as float64), so orders must be bit-exact and, the
    rounded preset times still being multiples of 2**-30 s, so must every float64 output; against
    the unrounded float64 samples the makespans agree within the float32 bound of 1e-3 relative.
    Includes samples with zero transfer times (the general TAC kernel) and per-sample orders."""
    makers = dict(SMALL)
    makers.update(EXTRA)
    d, h, dep = get(tt, name, makers.get(name))
    R = d.n_recv
    B = min(k, d.batch)
    op, rv = wl.timing_samples(d, 0, B)
    rng = np.random.default_rng(41)
    rv = rv.copy()
    rv[rng.random(rv.shape) < 0.02] = 0.0                      # a few zero-length transfers
    op32, rv32 = op.astype(np.float32), rv.astype(np.float32)
    op64, rv64 = op32.astype(np.float64), rv32.astype(np.float64)
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    eo, er, eP, eM = oracle.tac(dep, d.recv_ids, op64, rv64)
    exp = oracle.simulate(*args, eo, op64, rv64)
    got = tt.tac_simulate(h, cuda(op32), cuda(rv32), want_rank=True, want_sel=True)
    assert np.array_equal(got[0].cpu().numpy(), eo) and np.array_equal(got[1].cpu().numpy(), er)
    assert np.array_equal(got[2].cpu().numpy(), eP)
    gM = got[3].cpu().numpy()
    assert np.array_equal(np.isinf(gM), np.isinf(eM)) and np.array_equal(gM[np.isfinite(eM)], eM[np.isfinite(eM)])
    for a, b, nm in zip(got[4:], exp, "m E U L S".split()):
        assert np.array_equal(a.cpu().numpy(), b), f"{name}: fused {nm}"
    # the same samples unrounded: within the float32 bound
    ref = tt.simulate(h, got[0], cuda(op), cuda(rv))[0].cpu().numpy()
    assert np.allclose(got[4].cpu().numpy(), ref, rtol=1e-3, atol=0.0)
    # simulate alone: per-sample random orders and one shared order
    orders = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)
    for o in (orders, orders[0]):
        exp = oracle.simulate(*args, o, op64, rv64)
        got = tt.simulate(h, cuda(o), cuda(op32), cuda(rv32))
        for a, b, nm in zip(got, exp, "m E U L S".split()):
            assert np.array_equal(a.cpu().numpy(), b), f"{name}: simulate {nm}"


@pytest.mark.parametrize("name", ["tiny", "layered70", "resnet50", "r129", "slots5", "inception3"])
def test_times_that_are_not_quantised(tt, name):
    """Lognormal times as they come (sums round differently in different orders): float64 outputs
    within 1e-5 relative of the oracle's.  The simulation, the several-channel simulation and the
    search take no decision that rounding could turn (the search is compared through the makespan of
    the order it returns); TAC can, where two sums that are equal in exact arithmetic are formed in
    different ways, so its orders are compared sample by sample: an order that differs may differ
    only where the oracle's own round calls the choice a near tie (see tac_order_up_to_near_ties), and its
    makespan must be the one the oracle computes for it.  Two runs on the same inputs are equal byte for byte."""
    makers = dict(SMALL)
    makers.update(EXTRA)
    makers["slots5"] = CLASS_SLOTS[5]
    d, h, dep = get(tt, name, makers.get(name))
    R, B = d.n_recv, (8 if name == "inception3" else 48)
    rng = np.random.default_rng(77)
    op = rng.lognormal(np.log(1e-3), 0.5, size=(B, d.n_compute))
    rv = rng.lognormal(np.log(2e-3), 0.7, size=(B, R))
    gop, grv = cuda(op), cuda(rv)
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    orders = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)

    def close(got, exp, what):
        for a, b, nm in zip(got, exp, "m E U L S".split()):
            np.testing.assert_allclose(a.cpu().numpy(), b, rtol=RTOL, atol=1e-9 if nm in "ES" else 0.0,
                                       err_msg=f"{name}: {what} {nm}")

    close(tt.simulate(h, cuda(orders), gop, grv), oracle.simulate(*args, orders, op, rv), "simulate")
    chan = rng.integers(0, 3, size=R).astype(np.int32)
    close(tt.simulate_channels(h, 3, chan, cuda(orders), gop, grv),
          oracle.simulate_channels(*args, 3, chan, orders, op, rv), "three channels")
    got = tt.tac_simulate(h, gop, grv, want_rank=True, want_sel=True)
    again = tt.tac_simulate(h, gop, grv, want_rank=True, want_sel=True)
    for x, y in zip(got, again):
        assert torch.equal(x, y), f"{name}: two runs on the same unquantised inputs differ"
    go = got[0].cpu().numpy()
    assert np.array_equal(np.sort(go, axis=1), np.tile(np.arange(R, dtype=np.int32), (B, 1)))
    eo = oracle.tac(dep, d.recv_ids, op, rv)[0]
    same = (go == eo).all(axis=1)
    near = [tac_order_up_to_near_ties(oracle, d, dep, op[b], rv[b], go[b]) for b in np.nonzero(~same)[0]]
    print(f"[unquantised] {name}: {int(same.sum())} of {B} TAC orders equal to the oracle's; the others differ "
          f"at near ties only ({near} per sample)", flush=True)
    close(got[4:], oracle.simulate(*args, go, op, rv), "fused, under the order the GPU chose")
    moves = rng.integers(0, R, size=(40, 2)).astype(np.int32)
    best, mb, ms, acc = tt.order_search(h, cuda(orders), cuda(moves), gop, grv)
    bo = best.cpu().numpy()
    assert np.array_equal(np.sort(bo, axis=1), np.tile(np.arange(R, dtype=np.int32), (B, 1)))
    np.testing.assert_allclose(mb.cpu().numpy(), oracle.simulate(*args, bo, op, rv)[0], rtol=RTOL)
    np.testing.assert_allclose(ms.cpu().numpy(), oracle.simulate(*args, orders, op, rv)[0], rtol=RTOL)
    assert bool((mb <= ms).all())


def test_time_oracle_min(tt):
    """Minimum over measured runs, element by element against the oracle: even and odd lengths
    (two-element and one-element loads), one run, many runs, a batch of timing rows."""
    rng = np.random.default_rng(4)
    for K, n in ((5, 1000), (5, 1001), (1, 77), (2, 1), (9, 300001), (5, 0)):
        runs = rng.integers(1, 10**6, size=(K, n)).astype(np.float64) * wl.QUANTUM
        got = tt.time_oracle_min(cuda(runs)).cpu().numpy()
        assert np.array_equal(got, oracle.time_oracle_min(runs)), (K, n)
    d = wl.preset("resnet50")
    ops = np.stack([wl.timing_samples(d, 256 * k, 256 * k + 64)[0] for k in range(5)])      # [5][64][N]
    got = tt.time_oracle_min(cuda(ops)).cpu().numpy()
    assert got.shape == ops.shape[1:]
    assert np.array_equal(got.ravel(), oracle.time_oracle_min(ops.reshape(5, -1)))


def test_power_of_two_scaling_and_determinism(tt):
    d, h, dep = get(tt, "resnet50")
    op, rv = wl.timing_samples(d, 0, 64)
    a = tt.tac_simulate(h, cuda(op), cuda(rv), want_rank=True, want_sel=True)
    b = tt.tac_simulate(h, cuda(op), cuda(rv), want_rank=True, want_sel=True)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    c = tt.tac_simulate(h, cuda(op * 4), cuda(rv * 4), want_rank=True, want_sel=True)
    assert torch.equal(a[0], c[0])
    assert torch.equal(a[4] * 4, c[4]) and torch.equal(a[5], c[5]) and torch.equal(a[8], c[8])


# --------------------------------------------------------------------------
# full sizes, in the launch configuration the benchmark times
# --------------------------------------------------------------------------

def closed_form_shared(depb_comp, order, op, rv):
    """Makespan of every sample under one shared order, recomputed from the oracle's dep matrix
    alone: kappa of an op = last position among its recvs, A_k = time of the ops with kappa = k,
    makespan = max_k (F_k + A_k + ... + A_R) (see helpers.closed_form_makespan)."""
    import scipy.sparse as sp
    R = order.size
    N = depb_comp.shape[0]
    pos = np.zeros(R, dtype=np.int32)
    pos[order] = np.arange(1, R + 1, dtype=np.int32)
    kappa = np.zeros(N, dtype=np.int64)
    for n0 in range(0, N, 8192):
        blk = depb_comp[n0:n0 + 8192]
        kappa[n0:n0 + 8192] = (blk * pos[None, :]).max(axis=1) if R else 0
    onehot = sp.csr_matrix((np.ones(N), (np.arange(N), kappa)), shape=(N, R + 1))
    A = np.asarray((onehot.T @ op.T).T)
    F = np.concatenate([np.zeros((op.shape[0], 1)), np.cumsum(rv[:, order], axis=1)], axis=1)
    S = np.cumsum(A[:, ::-1], axis=1)[:, ::-1]
    return np.maximum((F + S).max(axis=1), F[:, -1])


def check_sampled_rounds(tt, d, dep, op_rows, rv_rows, orders, ks, tag, sel_P=None, sel_Mplus=None):
    """Rounds `ks` of every given sample: the oracle, started from the recvs that the GPU's own order
    has not removed before round k, must select what the GPU selected in round k (and, when the
    per-round outputs are given, with the same P and M+)."""
    for b in range(orders.shape[0]):
        print(f"[rounds] {tag}: sample {b}, {len(ks)} oracle rounds", flush=True)
        sel, eP, eM = oracle_rounds_after_prefix(dep, d.recv_ids, op_rows[b], rv_rows[b], orders[b], ks, threads=12)
        got = orders[b][list(ks)]
        assert np.array_equal(got, sel), f"{tag}: sample {b}: rounds {[k for k, a, e in zip(ks, got, sel) if a != e]} differ"
        if sel_P is not None:
            np.testing.assert_allclose(sel_P[b][sel], eP, rtol=RTOL, atol=0)
            gM = sel_Mplus[b][sel]
            assert np.array_equal(np.isinf(gM), np.isinf(eM))
            np.testing.assert_allclose(gM[np.isfinite(eM)], eM[np.isfinite(eM)], rtol=RTOL, atol=0)


STRESS_ROUNDS = list(range(16)) + [64, 512, 1024, 2048] + list(range(4080, 4096))


@pytest.mark.parametrize("name,B", [("resnet50", 65536), ("vgg16", 262144), ("inception3", 65536), ("stress", 4096)])
def test_full_batch_properties(tt, name, B):
    """Whole batch of the preset, in the launch configuration the benchmark times: every order is a
    permutation, L <= m <= U, sampled rows equal the oracle exactly (on the stress preset, whose
    4096 rounds per sample the oracle cannot run in full: sampled rounds of two rows, each started
    from the GPU's own prefix), and the makespans under the shared TIC order equal the closed form
    recomputed in numpy from the oracle's dep matrix on every sample."""
    d, h, dep = get(tt, name)
    assert B == d.batch
    print(f"[full] {name}: generating {B} samples", flush=True)
    op, rv = wl.timing_samples(d, 0, B)
    gop, grv = cuda(op), cuda(rv)
    print(f"[full] {name}: tac_simulate", flush=True)
    res = tt.tac_simulate(h, gop, grv, want_rank=True)
    order, rank = res[0], res[1]
    m, e, U, L, S = (x.cpu().numpy() for x in res[4:])
    R = d.n_recv
    srt = torch.sort(order.long(), dim=1).values
    assert torch.equal(srt, torch.arange(R, device="cuda").expand(B, R))
    del srt
    assert torch.equal(torch.gather(rank.long(), 1, order.long()), torch.arange(R, device="cuda").expand(B, R))
    assert (L <= m).all() and (m <= U).all() and (e >= 0).all() and (e <= 1).all()
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    if name == "stress":
        rows = [0, B - 1]
        go = order[rows].cpu().numpy()
        check_sampled_rounds(tt, d, dep, op[rows], rv[rows], go, STRESS_ROUNDS, name)
        exp = oracle.simulate(*args, go, op[rows], rv[rows])
        assert np.array_equal(m[rows], exp[0]) and np.array_equal(e[rows], exp[1])
    else:
        # sampled rows against the oracle
        rows = subset_rows(B, {"resnet50": 24, "vgg16": 256, "inception3": 32}[name])
        print(f"[full] {name}: oracle on {len(rows)} rows", flush=True)
        eo = oracle_tac_rows(dep, d.recv_ids, op[rows], rv[rows], threads=12)[0]
        assert np.array_equal(order[rows].cpu().numpy(), eo)
        exp = oracle.simulate(*args, eo, op[rows], rv[rows])
        assert np.array_equal(m[rows], exp[0]) and np.array_equal(e[rows], exp[1])
    # shared TIC order on the whole batch against the closed form
    print(f"[full] {name}: closed form on every sample", flush=True)
    tic_order = oracle.tic(dep, d.recv_ids)[1]
    m2 = tt.simulate(h, cuda(tic_order), gop, grv)[0].cpu().numpy()
    depb = dep_bool(dep, R)[d.compute_ids()]
    blk = 512 if name == "stress" else 8192
    for b0 in range(0, B, blk):
        ref = closed_form_shared(depb, tic_order, op[b0:b0 + blk], rv[b0:b0 + blk])
        assert np.array_equal(m2[b0:b0 + blk], ref)
    if R > 512 or h.n_classes > 512:
        return
    # order search on the whole batch from random orders: permutations, never worse than the start,
    # the makespan it reports is the one of the order it returns, sampled rows equal the oracle
    print(f"[full] {name}: order search", flush=True)
    rnd = wl.random_orders(d, 0, B)
    n_moves = 48 if name == "inception3" else 192
    moves = np.random.default_rng(3).integers(0, R, size=(n_moves, 2)).astype(np.int32)
    best, mb, ms, acc = tt.order_search(h, cuda(rnd), cuda(moves), gop, grv)
    assert torch.equal(torch.sort(best.long(), dim=1).values, torch.arange(R, device="cuda").expand(B, R))
    assert bool((mb <= ms).all()) and bool(((acc > 0) == (mb < ms)).all())
    assert torch.equal(tt.simulate(h, best, gop, grv)[0], mb)
    assert torch.equal(tt.simulate(h, cuda(rnd), gop, grv)[0], ms)
    rows = subset_rows(B, {"resnet50": 12, "vgg16": 64, "inception3": 3}[name])
    exp = oracle.order_search(*args, rnd[rows], moves, op[rows], rv[rows])
    for a, b_ in zip((best, mb, ms, acc), exp):
        assert np.array_equal(a[rows].cpu().numpy(), b_)


def test_stress_both_kernels_sampled_rounds(tt):
    """Preset 5, two samples, through both TAC kernels that serve a graph of this size: the call
    without per-round outputs and the call with them (sel_P, sel_Mplus).  The oracle cannot run
    all 4096 rounds of Algorithm 3 on a 100 000-op graph in reasonable time, so sampled rounds
    are compared, each started from the GPU's own prefix; the two GPU orders must be equal to
    each other in full, and the simulation under them equal to the oracle's event-driven one."""
    d, h, dep = get(tt, "stress")
    rows = [1, 2049]
    op, rv = wl.sample_rows(d, rows)
    print("[stress] GPU TAC on 2 samples, without and with per-round outputs", flush=True)
    res = tt.tac_simulate(h, cuda(op), cuda(rv), want_rank=True)
    order = res[0].cpu().numpy()
    assert np.array_equal(np.sort(order, axis=1), np.tile(np.arange(d.n_recv), (2, 1)))
    res2 = tt.tac_simulate(h, cuda(op), cuda(rv), want_rank=True, want_sel=True)
    assert np.array_equal(res2[0].cpu().numpy(), order)
    assert np.array_equal(res2[1].cpu().numpy(), res[1].cpu().numpy())
    ks = list(range(8)) + [300, 1500, 3000] + list(range(4090, 4096))
    check_sampled_rounds(tt, d, dep, op, rv, order, ks, "stress/sel", res2[2].cpu().numpy(), res2[3].cpu().numpy())
    print("[stress] simulate", flush=True)
    exp = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, order, op, rv)
    got = [x.cpu().numpy() for x in tt.simulate(h, cuda(order), cuda(op), cuda(rv))]
    for a, b in zip(got, exp):
        assert np.array_equal(a, b)
    assert np.array_equal(res[4].cpu().numpy(), exp[0]) and np.array_equal(res2[4].cpu().numpy(), exp[0])
    tic_order = oracle.tic(dep, d.recv_ids)[1]
    exp2 = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, tic_order, op, rv)
    got2 = tt.simulate(h, cuda(tic_order), cuda(op), cuda(rv))
    assert np.array_equal(got2[0].cpu().numpy(), exp2[0])


# --------------------------------------------------------------------------
# graphs with thousands of classes: the TAC kernels that serve the stress preset, on graphs small
# enough for the oracle to run every round
# --------------------------------------------------------------------------

# layered graphs whose numbers of classes need four, five, six and eight class slots per lane in the
# one-wave-per-sample kernels (seven: inception3; one to three: the small graphs above)
CLASS_SLOTS = {
    # (enough recvs for the simulation kernel with one wave per sample: 32 per class slot)
    4: lambda: wl.layered_dag(32, levels=10, width=24, fan_in=(1, 3), back=3, n_recv=130, attach=(1, 3), name="slots4"),
    5: lambda: wl.layered_dag(33, levels=11, width=28, fan_in=(1, 3), back=3, n_recv=165, attach=(1, 3), name="slots5"),
    6: lambda: wl.layered_dag(35, levels=13, width=33, fan_in=(1, 3), back=3, n_recv=200, attach=(1, 3), name="slots6"),
    8: lambda: wl.layered_dag(39, levels=15, width=40, fan_in=(1, 3), back=3, n_recv=260, attach=(1, 3), name="slots8"),
}


@pytest.mark.parametrize("slots", list(CLASS_SLOTS))
def test_every_number_of_class_slots(tt, slots):
    """The one-wave-per-sample kernels are instantiated per number of class slots per lane: TAC with the fused
    simulation, the simulation under given orders, several channels and the order search on graphs that need
    four, five, six and eight of them, each against the oracle."""
    name = f"slots{slots}"
    d, h, dep = get(tt, name, CLASS_SLOTS[slots])
    print(f"[slots] {name}: N={d.n_compute} R={d.n_recv} classes={h.n_classes}", flush=True)
    assert (h.n_classes + 63) // 64 == slots
    R, B = d.n_recv, 12
    assert R >= 32 * slots
    op, rv = wl.timing_samples(d, 0, B)
    run_tac_sim_parity(tt, d, h, dep, op, rv, name)
    rng = np.random.default_rng(61)
    orders = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)
    gop, grv, gord = cuda(op), cuda(rv), cuda(orders)
    args = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    for C, chan in ((3, np.arange(R) % 3), (4, rng.integers(0, 4, size=R))):
        chan = chan.astype(np.int32)
        exp = oracle.simulate_channels(*args, C, chan, orders, op, rv)
        got = tt.simulate_channels(h, C, chan, gord, gop, grv)
        for a, b, nm in zip(got, exp, "m E U L S".split()):
            assert np.array_equal(a.cpu().numpy(), b), f"{name}: {C} channels, {nm}"
    moves = rng.integers(0, R, size=(60, 2)).astype(np.int32)
    exp = oracle.order_search(*args, orders, moves, op, rv)
    got = tt.order_search(h, gord, cuda(moves), gop, grv)
    for a, b, nm in zip(got, exp, ("best_order", "best_makespan", "start_makespan", "n_accepted")):
        assert np.array_equal(a.cpu().numpy(), b), f"{name}: {nm}"


@pytest.mark.parametrize("slots", [4, 6, 8])
def test_ties_and_zero_times_with_many_class_slots(tt, slots):
    """The paths that graphs with four or more class slots per lane take for three or four members of Q:
    times from a handful of values (exact ties in the comparator, several pointers at one recv), zero
    compute times (classes that never point) and zero transfer times (the literal path), against the oracle."""
    name = f"slots{slots}"
    d, h, dep = get(tt, name, CLASS_SLOTS[slots])
    rng = np.random.default_rng(70 + slots)
    B = 40
    op = rng.integers(0, 4, size=(B, d.n_compute)).astype(np.float64) * 0.25
    rv = rng.integers(1, 4, size=(B, d.n_recv)).astype(np.float64) * 0.25
    run_tac_sim_parity(tt, d, h, dep, op, rv, name + "/ties")
    op1 = rng.integers(1, 9, size=(B, d.n_compute)).astype(np.float64) * 0.125     # no zero class times: many pointers
    run_tac_sim_parity(tt, d, h, dep, op1, rv, name + "/ties, positive times")
    rv0 = rv.copy()
    rv0[rng.random(rv0.shape) < 0.1] = 0.0
    run_tac_sim_parity(tt, d, h, dep, op[:8], rv0[:8], name + "/zero-transfers")


MANY_CLASSES = {
    # per-sample state beyond what one workgroup's LDS holds (about 9 600 classes, 160 recvs)
    "mid_stress": lambda: wl.stress_dag(levels=50, width=400, n_recv=160, seed=31, batch=8),
    # three words per row, recv count off the word boundary
    "mid_stress_w3": lambda: wl.stress_dag(levels=30, width=300, n_recv=150, seed=32, batch=8),
}


@pytest.mark.parametrize("name", list(MANY_CLASSES))
def test_many_classes_full_rounds(tt, name):
    d, h, dep = get(tt, name, MANY_CLASSES[name])
    print(f"[many] {name}: N={d.n_compute} R={d.n_recv} classes={h.n_classes}", flush=True)
    assert h.n_classes > 4000
    op, rv = wl.timing_samples(d, 0, 5)
    run_tac_sim_parity(tt, d, h, dep, op, rv, name)
    # exact ties in the comparator, zero-time ops, and transfer times of zero (the literal path)
    rng = np.random.default_rng(5)
    op3 = rng.integers(0, 4, size=(3, d.n_compute)).astype(np.float64) * 0.25
    rv3 = rng.integers(1, 4, size=(3, d.n_recv)).astype(np.float64) * 0.25
    run_tac_sim_parity(tt, d, h, dep, op3, rv3, name + "/ties")
    rv0 = rv3.copy()
    rv0[rng.random(rv0.shape) < 0.2] = 0.0
    run_tac_sim_parity(tt, d, h, dep, op3, rv0, name + "/zero-transfers")


@pytest.mark.parametrize("name", ["layered70", "tiny", "r129", "mid_stress_w3"])
def test_zero_transfer_times_that_are_not_quantised(tt, name):
    """Lognormal times as they come, a fifth of the transfer times set to zero: the samples take the
    literal selection path, in which M of a class is the fresh ascending sum over its outstanding
    recvs, as in Algorithm 1 (a class whose outstanding recvs all have time zero has M = 0 exactly,
    and M+ = 0 of its recvs ties exactly with other zeros).  Orders, ranks and the infinite entries
    of M+ must equal the oracle's."""
    makers = dict(SMALL)
    makers.update(EXTRA)
    makers.update(MANY_CLASSES)
    d, h, dep = get(tt, name, makers.get(name))
    R, B = d.n_recv, 4 if name.startswith("mid") else 40
    rng = np.random.default_rng(123)
    op = rng.lognormal(np.log(1e-3), 0.5, size=(B, d.n_compute))
    rv = rng.lognormal(np.log(2e-3), 0.7, size=(B, R))
    rv[rng.random(rv.shape) < 0.2] = 0.0
    rv[0, :] = 0.0                                  # every transfer time zero
    eo, er, eP, eM = oracle_tac_rows(dep, d.recv_ids, op, rv, threads=4)
    for want_sel in (True, False):
        got = tt.tac_simulate(h, cuda(op), cuda(rv), want_rank=True, want_sel=want_sel)
        go = got[0].cpu().numpy()
        diff = np.flatnonzero((go != eo).any(axis=1))
        assert diff.size == 0, f"{name}: samples {diff.tolist()} differ (want_sel={want_sel})"
        assert np.array_equal(got[1].cpu().numpy(), er)
        if want_sel:
            gM = got[3].cpu().numpy()
            assert np.array_equal(np.isinf(gM), np.isinf(eM))
            np.testing.assert_allclose(gM[np.isfinite(eM)], eM[np.isfinite(eM)], rtol=RTOL, atol=0)
            np.testing.assert_allclose(got[2].cpu().numpy(), eP, rtol=RTOL, atol=0)
        exp = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, eo, op, rv)
        for a, b, nm in zip(got[4:], exp, "m E U L S".split()):
            np.testing.assert_allclose(a.cpu().numpy(), b, rtol=RTOL, atol=1e-9 if nm in "ES" else 0.0)


def test_class_grouping_on_the_device_equals_the_host_grouping(tt):
    """Large graphs are grouped into classes of equal dependency rows from hashes formed on the device (the rows
    stay there); the same graph grouped on the host from the rows themselves must give the same classes and,
    through them, the same TAC orders and iteration metrics."""
    d = wl.preset("stress")
    assert d.n_ops * d.words * 8 >= 8 << 20
    h_dev = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    os.environ["TICTAC_GROUP_ON_HOST"] = "1"
    try:
        h_host = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    finally:
        del os.environ["TICTAC_GROUP_ON_HOST"]
    assert h_dev.n_classes == h_host.n_classes == 60567
    op, rv = wl.timing_samples(d, 0, 2)
    a = tt.tac_simulate(h_dev, cuda(op), cuda(rv), want_rank=True)
    b = tt.tac_simulate(h_host, cuda(op), cuda(rv), want_rank=True)
    for x, y in zip(a, b):
        if x is not None:
            assert torch.equal(x, y)
    pa, pb = tt.tic_priority(h_dev), tt.tic_priority(h_host)
    for x, y in zip(pa, pb):
        assert torch.equal(x, y)
    h_dev.close()
    h_host.close()
