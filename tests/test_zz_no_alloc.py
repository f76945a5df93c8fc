"""tictac_tac_simulate_noalloc, the entry point that allocates nothing, against tictac_tac_simulate:
equal outputs on two calls in a row, the second on a smaller batch whose samples with a transfer time
of zero (the ones the call flags in its static array) sit elsewhere than in the first."""

import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1803_03288_amd import workloads as wl


def test_no_alloc_entry_point_equals_tac_simulate():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1803_03288_amd import binding as tt
    tt.lib()
    d = wl.preset("resnet50")
    h = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
    R = d.n_recv
    rng = np.random.default_rng(5)
    for B, zero_from in ((700, 0), (130, 60)):
        op, rv = wl.timing_samples(d, 1000, 1000 + B)
        rv = rv.copy()
        z = np.zeros(B, dtype=bool)
        z[zero_from:zero_from + 40:3] = True                  # these samples get a few transfer times of zero
        rv[np.outer(z, rng.random(R) < 0.1)] = 0.0
        gop, grv = torch.from_numpy(op).cuda(), torch.from_numpy(rv).cuda()
        ref = tt.tac_simulate(h, gop, grv, want_rank=True)
        out = (torch.full((B, R), -7, dtype=torch.int32, device="cuda"), torch.full((B, R), -7, dtype=torch.int32, device="cuda")) + \
              tuple(torch.full((B,), -7.0, dtype=torch.float64, device="cuda") for _ in range(5))
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        got = tt.tac_simulate_noalloc(h, gop, grv, out)
        torch.cuda.synchronize()
        if B != 700:        # (the first call of a process loads the kernels' code; from the second on nothing may change)
            assert torch.cuda.mem_get_info()[0] == free_before
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
        for a, b in zip(got[2:], ref[4:]):
            assert torch.equal(a, b)
    # sizes beyond what the call serves: an error, nothing written
    L = tt.lib()
    rc = L.tictac_tac_simulate_noalloc(h._h, ctypes.c_int32((1 << 20) + 1), ctypes.c_void_p(8), ctypes.c_void_p(8),
                                       ctypes.c_void_p(8), None, None, None, None, None, None, None)
    assert rc == -9 and b"2^20" not in L.tictac_last_error() and b"1048576" in L.tictac_last_error()
    ds = wl.stress_dag(levels=30, width=300, n_recv=150, seed=32, batch=8)
    hs = tt.build_deps(ds.n_ops, ds.row_ptr, ds.col_idx, ds.recv_ids)
    ops, rvs = wl.timing_samples(ds, 0, 2)
    outs = (torch.full((2, 150), -7, dtype=torch.int32, device="cuda"), None) + \
           tuple(torch.full((2,), -7.0, dtype=torch.float64, device="cuda") for _ in range(5))
    with pytest.raises(tt.TicTacError) as e:
        tt.tac_simulate_noalloc(hs, torch.from_numpy(ops).cuda(), torch.from_numpy(rvs).cuda(), outs)
    assert e.value.code == -9
    assert int((outs[0] != -7).sum()) == 0 and float(outs[2].max()) == -7.0
