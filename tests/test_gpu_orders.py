"""Orders handed to the simulations and to the search must be permutations of the recvs (Sec. 3.2: the order
of the transfers).  The calls are asynchronous, so the device checks every order and raises a flag of the
handle, which ``tictac_dag_check_orders`` reports as TICTAC_ERR_BAD_ORDER and lowers.  Entries out of range
are skipped by the kernels: nothing is read or written out of bounds, and the samples whose orders are
valid come out as without the bad ones."""

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1803_03288_amd import workloads as wl


@pytest.fixture(scope="module")
def tt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1803_03288_amd import binding
    binding.lib()
    return binding


def cuda(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


GRAPHS = {
    "tiny": lambda: wl.preset("tiny"),
    "resnet50": lambda: wl.preset("resnet50"),
    "layered70": lambda: wl.layered_dag(11, levels=9, width=7, fan_in=(1, 3), back=3, n_recv=70, attach=(1, 3)),
}


def expect_bad(tt, h):
    with pytest.raises(tt.TicTacError) as e:
        h.check_orders()
    assert e.value.code == -6
    h.check_orders()            # the flag was lowered


@pytest.mark.parametrize("name", list(GRAPHS))
def test_orders_are_checked_on_the_device(tt, name):
    d = GRAPHS[name]()
    R, B = d.n_recv, 37
    h = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    rng = np.random.default_rng(3)
    op, rv = wl.timing_samples(d, 0, B)
    gop, grv = cuda(op), cuda(rv)
    orders = np.stack([rng.permutation(R) for _ in range(B)]).astype(np.int32)
    chan = rng.integers(0, 2, size=R).astype(np.int32)
    moves = cuda(rng.integers(0, R, size=(8, 2)).astype(np.int32))
    searchable = R <= 512 and h.n_classes <= 512

    clean = [x.cpu().numpy() for x in tt.simulate(h, cuda(orders), gop, grv)]
    tt.simulate(h, cuda(orders[0]), gop, grv)
    tt.simulate_channels(h, 2, chan, cuda(orders), gop, grv)
    if searchable:
        tt.order_search(h, cuda(orders), moves, gop, grv)
    h.check_orders()            # nothing wrong so far

    bad_rows = {5: "twice", 11: "negative", 20: "too large", 36: "far too large"}
    broken = orders.copy()
    broken[5, 3] = broken[5, 9]
    broken[11, 0] = -1
    broken[20, R - 1] = R
    broken[36, R // 2] = 2**31 - 1
    good = np.array([b for b in range(B) if b not in bad_rows])

    got = [x.cpu().numpy() for x in tt.simulate(h, cuda(broken), gop, grv)]
    expect_bad(tt, h)
    for a, b in zip(got, clean):
        assert np.array_equal(a[good], b[good]), f"{name}: a valid sample changed next to an invalid one"

    for row in bad_rows:
        tt.simulate(h, cuda(broken[row]), gop, grv)         # one order for every sample
        expect_bad(tt, h)
    tt.simulate_channels(h, 2, chan, cuda(broken), gop, grv)
    expect_bad(tt, h)
    if searchable:
        tt.order_search(h, cuda(broken), moves, gop, grv)
        expect_bad(tt, h)
    op32, rv32 = cuda(op.astype(np.float32)), cuda(rv.astype(np.float32))
    tt.simulate(h, cuda(broken), op32, rv32)
    expect_bad(tt, h)

    # several calls, one of them bad: the flag stays up until it is asked for
    tt.simulate(h, cuda(broken), gop, grv)
    tt.simulate(h, cuda(orders), gop, grv)
    expect_bad(tt, h)
    # the orders TAC produces pass
    o = tt.tac_simulate(h, gop, grv)[0]
    tt.simulate(h, o, gop, grv)
    h.check_orders()
    h.close()
