"""Seeded synthetic inputs: computational DAGs with root ``recv`` ops and batches
of per-op timing samples.

This module only *draws inputs*.  It contains none of the scheduling method's
arithmetic (no dependency sets, priorities or makespans), so that the CPU
checker and the GPU library can both be fed from it without sharing any code of
the method itself.

The paper (Sec. 3.1) takes as input a partitioned graph, whose communication
ops (``recv``) are roots of the worker DAG (Sec. 2.2), and a time oracle
``Time(op)``.  The graphs of its evaluation (Appendix A, Table 1: ResNet-50 v2,
VGG-16, Inception v3, ...) are TensorFlow graphs that are not available; the
presets below are synthetic DAGs of the same shape (parameter counts, chain /
residual / multi-branch structure, forward or forward+backward) and every
timing sample stands in for one traced iteration.

Conventions
-----------
* A DAG is a predecessor CSR over op ids ``0..n_ops-1`` plus ``recv_ids``:
  ``recv_ids[i]`` is the op id of recv ``i``.  The presets number the recvs
  first (``recv_ids = 0..R-1``) and the compute ops topologically after them.
* ``op_time`` is ``[B][N]`` float64, column ``j`` = the j-th compute op in
  ascending op id; ``recv_time`` is ``[B][R]``, column ``i`` = recv ``i``.
* Every time is rounded to a multiple of 2**-30 s and clamped to at least
  2**-30 s, so that all partial sums that the method forms are exact in
  float64 whatever the order of summation.
* Random numbers: ``numpy.random.Generator(PCG64(SeedSequence([seed, stream,
  chunk])))``.  Stream 0 draws the structure, 1 the parameter sizes, 2 the
  compute times, 3 the transfer times; times are drawn in chunks of
  ``CHUNK`` samples, each chunk from its own sequence, so that any range of
  samples can be produced without drawing the ones before it.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

QUANTUM = 2.0 ** -30          # seconds
LINK_BITS_PER_S = 1.0e10      # 10 Gb/s link of every preset
CHUNK = 256                   # samples per independently seeded chunk

_STREAM_STRUCT, _STREAM_SIZE, _STREAM_OP, _STREAM_RECV, _STREAM_ORDER = 0, 1, 2, 3, 4


def _rng(seed: int, stream: int, chunk: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, chunk])))


def quantise(t: np.ndarray) -> np.ndarray:
    """Round to the nearest multiple of 2**-30 s, at least one quantum."""
    q = np.rint(np.asarray(t, dtype=np.float64) * (1.0 / QUANTUM))
    np.maximum(q, 1.0, out=q)
    q *= QUANTUM
    return q


@dataclass
class Dag:
    """A worker DAG (predecessor CSR) and the timing model of its ops."""

    name: str
    n_ops: int
    row_ptr: np.ndarray          # int32 [n_ops + 1]
    col_idx: np.ndarray          # int32 [E], predecessors of op v in row_ptr[v]:row_ptr[v+1]
    recv_ids: np.ndarray         # int32 [R]
    op_median: np.ndarray        # float64 [N] seconds (mean for 'exponential')
    recv_bytes: np.ndarray       # float64 [R]
    op_dist: str = "lognormal"   # 'lognormal' | 'exponential'
    op_sigma: float = 0.3
    recv_sigma: float = 0.2
    seed: int = 0
    batch: int = 1024            # B of the preset
    op_kind: List[str] = field(default_factory=list)  # per compute op, informative only

    @property
    def n_recv(self) -> int:
        return int(self.recv_ids.shape[0])

    @property
    def n_compute(self) -> int:
        return self.n_ops - self.n_recv

    @property
    def n_edges(self) -> int:
        return int(self.col_idx.shape[0])

    @property
    def words(self) -> int:
        return (self.n_recv + 63) // 64

    def compute_ids(self) -> np.ndarray:
        """Op ids of the compute ops in ascending order (column order of op_time)."""
        mask = np.ones(self.n_ops, dtype=bool)
        mask[self.recv_ids] = False
        return np.nonzero(mask)[0].astype(np.int32)

    def recv_base_time(self) -> np.ndarray:
        """Transfer time of each recv on the dedicated 10 Gb/s link, seconds."""
        return 8.0 * self.recv_bytes / LINK_BITS_PER_S


class _Builder:
    """Collects ops in creation order (predecessors must already exist) and
    renumbers them recvs-first at the end."""

    def __init__(self) -> None:
        self.is_recv: List[bool] = []
        self.preds: List[Tuple[int, ...]] = []
        self.median: List[float] = []     # compute ops only (0 for recvs)
        self.size: List[float] = []       # recvs only (0 for compute ops)
        self.kind: List[str] = []

    def recv(self, nbytes: float, kind: str = "param") -> int:
        self.is_recv.append(True)
        self.preds.append(())
        self.median.append(0.0)
        self.size.append(float(nbytes))
        self.kind.append(kind)
        return len(self.is_recv) - 1

    def op(self, preds: Sequence[int], median: float, kind: str = "op") -> int:
        p = tuple(dict.fromkeys(int(x) for x in preds))  # distinct, order kept
        for x in p:
            assert 0 <= x < len(self.is_recv)
        self.is_recv.append(False)
        self.preds.append(p)
        self.median.append(float(median))
        self.size.append(0.0)
        self.kind.append(kind)
        return len(self.is_recv) - 1

    def chain(self, first_preds: Sequence[int], medians: Sequence[float], kind: str,
              feed: Optional[dict] = None) -> int:
        """A chain of ops; ``feed[k]`` lists extra predecessors (recvs) of the k-th op."""
        feed = feed or {}
        prev: Optional[int] = None
        for k, m in enumerate(medians):
            p = list(first_preds) if prev is None else [prev]
            p += list(feed.get(k, ()))
            prev = self.op(p, m, kind)
        assert prev is not None
        return prev

    def finish(self, name: str, **kw) -> Dag:
        n = len(self.is_recv)
        is_recv = np.array(self.is_recv, dtype=bool)
        old_recv = np.nonzero(is_recv)[0]
        old_comp = np.nonzero(~is_recv)[0]
        new_id = np.empty(n, dtype=np.int64)
        new_id[old_recv] = np.arange(old_recv.size)
        new_id[old_comp] = old_recv.size + np.arange(old_comp.size)
        order = np.concatenate([old_recv, old_comp])
        row_ptr = np.zeros(n + 1, dtype=np.int64)
        cols: List[int] = []
        for k, old in enumerate(order):
            ps = self.preds[old]
            cols.extend(int(new_id[p]) for p in ps)
            row_ptr[k + 1] = len(cols)
        return Dag(
            name=name,
            n_ops=n,
            row_ptr=row_ptr.astype(np.int32),
            col_idx=np.array(cols, dtype=np.int32),
            recv_ids=np.arange(old_recv.size, dtype=np.int32),
            op_median=np.array([self.median[o] for o in old_comp], dtype=np.float64),
            recv_bytes=np.array([self.size[o] for o in old_recv], dtype=np.float64),
            op_kind=[self.kind[o] for o in old_comp],
            **kw,
        )


# --------------------------------------------------------------------------
# timing samples
# --------------------------------------------------------------------------

def timing_samples(dag: Dag, b0: int = 0, b1: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Rows ``b0..b1-1`` of the preset's ``op_time [B][N]`` and ``recv_time [B][R]``."""
    if b1 is None:
        b1 = dag.batch
    assert 0 <= b0 <= b1
    N, R = dag.n_compute, dag.n_recv
    op = np.empty((b1 - b0, N), dtype=np.float64)
    rv = np.empty((b1 - b0, R), dtype=np.float64)
    base = dag.recv_base_time()
    c0, c1 = b0 // CHUNK, (b1 + CHUNK - 1) // CHUNK
    for c in range(c0, c1):
        lo, hi = max(b0, c * CHUNK), min(b1, (c + 1) * CHUNK)
        if hi <= lo:
            continue
        g_op, g_rv = _rng(dag.seed, _STREAM_OP, c), _rng(dag.seed, _STREAM_RECV, c)
        if dag.op_dist == "lognormal":
            z = g_op.standard_normal((CHUNK, N))
            blk = dag.op_median[None, :] * np.exp(dag.op_sigma * z)
        elif dag.op_dist == "exponential":
            blk = dag.op_median[None, :] * g_op.standard_exponential((CHUNK, N))
        else:
            raise ValueError(dag.op_dist)
        zr = g_rv.standard_normal((CHUNK, R))
        blk_r = base[None, :] * np.exp(dag.recv_sigma * zr)
        s = slice(lo - c * CHUNK, hi - c * CHUNK)
        op[lo - b0:hi - b0] = quantise(blk[s])
        rv[lo - b0:hi - b0] = quantise(blk_r[s])
    return op, rv


def random_orders(dag: Dag, b0: int = 0, b1: Optional[int] = None) -> np.ndarray:
    """Rows ``b0..b1-1`` of ``[B][R]`` int32: one uniformly random transfer order per sample, the
    stand-in for a system that imposes no order (every iteration and worker sees another one)."""
    if b1 is None:
        b1 = dag.batch
    assert 0 <= b0 <= b1
    R = dag.n_recv
    out = np.empty((b1 - b0, R), dtype=np.int32)
    for c in range(b0 // CHUNK, (b1 + CHUNK - 1) // CHUNK):
        lo, hi = max(b0, c * CHUNK), min(b1, (c + 1) * CHUNK)
        if hi <= lo:
            continue
        keys = _rng(dag.seed, _STREAM_ORDER, c).random((CHUNK, R))
        blk = np.argsort(keys, axis=1, kind="stable").astype(np.int32)
        out[lo - b0:hi - b0] = blk[lo - c * CHUNK:hi - c * CHUNK]
    return out


def sample_rows(dag: Dag, rows: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Selected rows of the preset's timing arrays (any order, any subset)."""
    rows = [int(r) for r in rows]
    op = np.empty((len(rows), dag.n_compute), dtype=np.float64)
    rv = np.empty((len(rows), dag.n_recv), dtype=np.float64)
    cache: dict = {}
    for k, r in enumerate(rows):
        c = r // CHUNK
        if c not in cache:
            cache.clear()
            cache[c] = timing_samples(dag, c * CHUNK, (c + 1) * CHUNK)
        o, v = cache[c]
        op[k], rv[k] = o[r - c * CHUNK], v[r - c * CHUNK]
    return op, rv


# --------------------------------------------------------------------------
# small structural families used by the tests
# --------------------------------------------------------------------------

def layered_dag(seed: int, levels: int, width: int, fan_in: Tuple[int, int], back: int,
                n_recv: int, attach: Tuple[int, int], name: str = "layered",
                op_median: float = 1e-3, size_range: Tuple[float, float] = (1e3, 4e6),
                size_log: bool = False, **kw) -> Dag:
    """``levels`` x ``width`` compute ops; an op of level >= 1 has U{fan_in} distinct
    predecessors drawn from the previous ``back`` levels; each recv feeds U{attach}
    distinct, uniformly chosen compute ops."""
    g = _rng(seed, _STREAM_STRUCT)
    gs = _rng(seed, _STREAM_SIZE)
    N = levels * width
    comp_preds: List[List[int]] = [[] for _ in range(N)]
    for lv in range(1, levels):
        lo = max(0, lv - back) * width
        hi = lv * width
        for k in range(width):
            f = int(g.integers(fan_in[0], fan_in[1] + 1))
            f = min(f, hi - lo)
            comp_preds[lv * width + k] = sorted(int(x) for x in g.choice(hi - lo, size=f, replace=False) + lo)
    recv_to: List[List[int]] = []
    for _ in range(n_recv):
        a = int(g.integers(attach[0], attach[1] + 1))
        recv_to.append([int(x) for x in g.choice(N, size=min(a, N), replace=False)])
    if size_log:
        sizes = np.exp(gs.uniform(np.log(size_range[0]), np.log(size_range[1]), size=n_recv))
    else:
        sizes = gs.uniform(size_range[0], size_range[1], size=n_recv)
    # ids: recvs 0..R-1, compute op c -> R + c
    R = n_recv
    extra: List[List[int]] = [[] for _ in range(N)]
    for i, tos in enumerate(recv_to):
        for c in tos:
            extra[c].append(i)
    row_ptr = np.zeros(R + N + 1, dtype=np.int64)
    cols: List[int] = []
    for c in range(N):
        cols.extend(sorted(extra[c]))
        cols.extend(R + p for p in comp_preds[c])
        row_ptr[R + c + 1] = len(cols)
    return Dag(name=name, n_ops=R + N, row_ptr=row_ptr.astype(np.int32),
               col_idx=np.array(cols, dtype=np.int32),
               recv_ids=np.arange(R, dtype=np.int32),
               op_median=np.full(N, op_median, dtype=np.float64),
               recv_bytes=np.rint(sizes).astype(np.float64), seed=seed, **kw)


def deep_narrow_dag(seed: int, levels: int, width: int, n_recv: int, name: str = "deep_narrow") -> Dag:
    """``levels`` x ``width`` compute ops; op (lv, k) depends on op (lv-1, k) and on one op drawn
    uniformly from all earlier levels (so most edges span many levels); each recv feeds one
    uniformly chosen compute op.  Deep, narrow, with long edges."""
    g = _rng(seed, _STREAM_STRUCT)
    gs = _rng(seed, _STREAM_SIZE)
    N, R = levels * width, n_recv
    extra: List[List[int]] = [[] for _ in range(N)]
    for i in range(R):
        extra[int(g.integers(0, N))].append(i)
    row_ptr = np.zeros(R + N + 1, dtype=np.int64)
    cols: List[int] = []
    for lv in range(levels):
        for k in range(width):
            c = lv * width + k
            cols.extend(sorted(extra[c]))
            if lv >= 1:
                far = int(g.integers(0, lv * width))
                cols.extend(sorted({R + (lv - 1) * width + k, R + far}))
            row_ptr[R + c + 1] = len(cols)
    sizes = gs.uniform(1e3, 4e6, size=R)
    return Dag(name=name, n_ops=R + N, row_ptr=row_ptr.astype(np.int32),
               col_idx=np.array(cols, dtype=np.int32), recv_ids=np.arange(R, dtype=np.int32),
               op_median=np.full(N, 1e-3, dtype=np.float64), recv_bytes=np.rint(sizes).astype(np.float64), seed=seed)


def chain_dag(n_recv: int, seed: int = 0, name: str = "chain") -> Dag:
    """``c_1 <- r_1``; ``c_k <- {c_{k-1}, r_k}``: a layer-by-layer model."""
    b = _Builder()
    rs = [b.recv(1e5 * (1 + (k % 3))) for k in range(n_recv)]
    prev: Optional[int] = None
    for k in range(n_recv):
        prev = b.op(([prev] if prev is not None else []) + [rs[k]], 1e-3, "layer")
    return b.finish(name, seed=seed, batch=8)


def independent_jobs_dag(n_recv: int, seed: int = 0) -> Dag:
    """recv ``i`` feeds one private compute op ``i``; nothing else (a two-machine flow shop)."""
    b = _Builder()
    rs = [b.recv(1e5) for _ in range(n_recv)]
    for r in rs:
        b.op([r], 1e-3, "job")
    return b.finish("jobs", seed=seed, batch=8)


def funnel_dag(n_recv: int, n_compute: int, seed: int = 0) -> Dag:
    """Every recv feeds one root compute op from which every other compute op descends."""
    b = _Builder()
    rs = [b.recv(1e5) for _ in range(n_recv)]
    prev = b.op(rs, 1e-3, "root")
    for _ in range(n_compute - 1):
        prev = b.op([prev], 1e-3, "op")
    return b.finish("funnel", seed=seed, batch=8)


def no_recv_dag(n_compute: int, seed: int = 0) -> Dag:
    b = _Builder()
    prev: Optional[int] = None
    for k in range(n_compute):
        prev = b.op([prev] if (prev is not None and k % 3) else [], 1e-3, "op")
    return b.finish("norecv", seed=seed, batch=8)


def toy_dag() -> Dag:
    """The toy graph of the paper's Fig. 1a: ``recv1 -> op1``; ``op2 <- {op1, recv2}``."""
    b = _Builder()
    r1, r2 = b.recv(1e5), b.recv(1e5)
    o1 = b.op([r1], 1e-3, "op1")
    b.op([o1, r2], 1e-3, "op2")
    return b.finish("toy", batch=8)


def case2_dag() -> Dag:
    """The second sample graph of Sec. 4.3: A and B feed one op; C, then D, join later."""
    b = _Builder()
    A, B_, C, D = b.recv(1e5), b.recv(2e5), b.recv(1e5), b.recv(1e5)
    o1 = b.op([A, B_], 1e-3, "op1")
    o2 = b.op([o1, C], 1e-3, "op2")
    b.op([o2, D], 1e-3, "op3")
    return b.finish("case2", batch=8)


def relabel(dag: Dag, seed: int) -> Tuple[Dag, np.ndarray]:
    """The same DAG under a random permutation of op ids (recv *indices* are kept:
    recv i stays recv i, at a new op id).  Returns the DAG and ``new_id[old_id]``.
    Column j of ``op_time`` refers to the j-th compute op in ascending *new* id, so
    timing arrays must be permuted with ``compute_column_map``."""
    g = _rng(seed, 7)
    n = dag.n_ops
    new_id = g.permutation(n).astype(np.int64)
    old_of_new = np.argsort(new_id)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    cols: List[int] = []
    for v_new in range(n):
        v_old = int(old_of_new[v_new])
        ps = dag.col_idx[dag.row_ptr[v_old]:dag.row_ptr[v_old + 1]]
        cols.extend(int(new_id[p]) for p in ps)
        row_ptr[v_new + 1] = len(cols)
    old_comp = dag.compute_ids()
    new_comp_sorted = np.sort(new_id[old_comp])
    # median per new compute column
    col_of_new = {int(v): j for j, v in enumerate(new_comp_sorted)}
    med = np.empty_like(dag.op_median)
    for j_old, v_old in enumerate(old_comp):
        med[col_of_new[int(new_id[v_old])]] = dag.op_median[j_old]
    out = Dag(name=dag.name + "-relabel", n_ops=n, row_ptr=row_ptr.astype(np.int32),
              col_idx=np.array(cols, dtype=np.int32),
              recv_ids=new_id[dag.recv_ids].astype(np.int32), op_median=med,
              recv_bytes=dag.recv_bytes.copy(), op_dist=dag.op_dist, op_sigma=dag.op_sigma,
              recv_sigma=dag.recv_sigma, seed=dag.seed, batch=dag.batch)
    return out, new_id


def compute_column_map(old: Dag, new: Dag, new_id: np.ndarray) -> np.ndarray:
    """``m[j_new] = j_old``: which old op_time column each new column takes."""
    old_comp = old.compute_ids()
    new_comp = new.compute_ids()
    col_of_new = {int(v): j for j, v in enumerate(new_comp)}
    m = np.empty(old_comp.size, dtype=np.int64)
    for j_old, v_old in enumerate(old_comp):
        m[col_of_new[int(new_id[v_old])]] = j_old
    return m


# --------------------------------------------------------------------------
# the five presets
# --------------------------------------------------------------------------

def tiny_dag() -> Dag:
    """Preset 1 (seed 0): 8 levels x 8 compute ops, fan-in U{1..3} from the previous
    level, 16 recvs each feeding U{1..2} compute ops; lognormal(ln 1 ms, 0.5) compute
    times; parameter sizes U[1 KB, 4 MB]."""
    return layered_dag(seed=0, levels=8, width=8, fan_in=(1, 3), back=1, n_recv=16,
                       attach=(1, 2), name="tiny", op_median=1e-3,
                       size_range=(1e3, 4e6), op_dist="lognormal", op_sigma=0.5,
                       recv_sigma=0.2, batch=1024)


def stress_dag(levels: int = 500, width: int = 200, n_recv: int = 4096, seed: int = 4,
               batch: int = 4096) -> Dag:
    """Preset 5 (seed 4): 500 levels x 200 compute ops, fan-in U{1..4} from the previous
    3 levels, 4096 recvs each attached to U{1..8} random compute ops; exponential
    compute times (mean 0.1 ms); parameter sizes log-uniform in [1 KB, 64 MB]."""
    return layered_dag(seed=seed, levels=levels, width=width, fan_in=(1, 4), back=3,
                       n_recv=n_recv, attach=(1, 8), name="stress", op_median=1e-4,
                       size_range=(1e3, 64e6), size_log=True, op_dist="exponential",
                       recv_sigma=0.2, batch=batch)


_AUX = 5e-5      # median of element-wise / bookkeeping ops, seconds
_BN = 1e-4       # median of the arithmetic ops of a batch normalisation
_FC = 3e-4


def _conv_unit(b: _Builder, x: int, W: int, med: float, pre: int, post: int, scale: float = 1.0) -> int:
    """Fine-grained expansion of a convolution: ``pre`` bookkeeping ops, the op that
    consumes the weight, ``post`` bookkeeping ops."""
    meds = [_AUX * scale] * pre + [med * scale] + [_AUX * scale] * post
    return b.chain([x], meds, "conv", feed={pre: [W]})


def _bn_unit(b: _Builder, x: int, gamma: int, beta: int, n: int, scale: float = 1.0) -> int:
    """Batch normalisation as a chain of ``n`` ops; the scale enters at op n-4, the
    offset at op n-2."""
    meds = [_AUX * scale] * n
    meds[n - 4] = _BN * scale
    meds[n - 2] = _BN * scale
    return b.chain([x], meds, "bn", feed={n - 4: [gamma], n - 2: [beta]})


def _lin_map(x: np.ndarray, lo: float, hi: float) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    if x.max() == x.min():
        return np.full_like(x, lo)
    return lo + (hi - lo) * (x - x.min()) / (x.max() - x.min())


def resnet50_dag() -> Dag:
    """Preset 2 (seed 1): forward graph shaped like ResNet-v2-50.  16 pre-activation
    bottleneck blocks in stages [3,4,6,3]; 161 parameter recvs: stem weight, per block
    3 conv weights + 3 x (scale, offset), 4 projection weights with (scale, offset),
    the final normalisation (scale, offset) and the classifier (weight, bias)."""
    b = _Builder()
    stages = [(3, 64, 256, 56), (4, 128, 512, 28), (6, 256, 1024, 14), (3, 512, 2048, 7)]
    cap = 8.0 * 2 ** 20

    # FLOPs of every conv first, to map them to medians in [0.5, 2] ms
    flops: List[float] = []
    flops.append(2 * 49 * 3 * 64 * 112 * 112)
    cin = 64
    for (nb, mid, out, hw) in stages:
        for k in range(nb):
            flops += [2 * cin * mid * hw * hw, 2 * 9 * mid * mid * hw * hw, 2 * mid * out * hw * hw]
            if k == 0:
                flops.append(2 * cin * out * hw * hw)
            cin = out
    med = list(_lin_map(np.array(flops), 5e-4, 2e-3))
    mi = iter(med)

    def P(nbytes: float) -> int:
        return b.recv(min(float(nbytes), cap))

    x = b.op([], _AUX, "input")
    x = _conv_unit(b, x, P(49 * 3 * 64 * 4), next(mi), 4, 4)
    x = b.chain([x], [_AUX, _AUX], "pool")
    cin = 64
    for (nb, mid, out, hw) in stages:
        for k in range(nb):
            skip = x
            h = _bn_unit(b, x, P(cin * 4), P(cin * 4), 9)
            h = b.chain([h], [_AUX, _AUX], "relu")
            pre = h
            h = _conv_unit(b, h, P(cin * mid * 4), next(mi), 4, 4)
            h = _bn_unit(b, h, P(mid * 4), P(mid * 4), 9)
            h = b.chain([h], [_AUX, _AUX], "relu")
            h = _conv_unit(b, h, P(9 * mid * mid * 4), next(mi), 4, 4)
            h = _bn_unit(b, h, P(mid * 4), P(mid * 4), 9)
            h = b.chain([h], [_AUX, _AUX], "relu")
            h = _conv_unit(b, h, P(mid * out * 4), next(mi), 4, 4)
            if k == 0:
                s = _conv_unit(b, pre, P(cin * out * 4), next(mi), 4, 4)
                skip = _bn_unit(b, s, P(out * 4), P(out * 4), 9)
            x = b.chain([h, skip], [_AUX, _AUX], "add")
            cin = out
    x = _bn_unit(b, x, P(2048 * 4), P(2048 * 4), 9)
    x = b.chain([x], [_AUX, _AUX], "relu")
    x = b.chain([x], [_AUX] * 3, "pool")
    x = b.chain([x], [_AUX, _FC, _AUX, _AUX, _AUX], "fc",
                feed={1: [P(2048 * 1000 * 4)], 3: [P(1000 * 4)]})
    b.chain([x], [_AUX] * 4, "softmax")
    return b.finish("resnet50", seed=1, batch=65536, op_dist="lognormal", op_sigma=0.3,
                    recv_sigma=0.2)


def vgg16_dag() -> Dag:
    """Preset 3 (seed 2): forward graph shaped like VGG-16, a pure chain of compute ops:
    13 x (conv, bias, relu), 5 pools, flatten, 3 fully connected layers, softmax.
    32 recvs = (weight, bias) x 16.  Medians = FLOPs at 10 TFLOP/s for a batch of 32
    images, at least 10 us."""
    b = _Builder()
    batch = 32.0
    floor = 1e-5

    def t(fl: float) -> float:
        return max(fl * batch / 1e13, floor)

    cfg = [(64, 224), (64, 224), "P", (128, 112), (128, 112), "P", (256, 56), (256, 56), (256, 56), "P",
           (512, 28), (512, 28), (512, 28), "P", (512, 14), (512, 14), (512, 14), "P"]
    x = b.op([], floor, "input")
    x = b.op([x], floor, "cast")
    cin = 3
    for c in cfg:
        if c == "P":
            x = b.op([x], floor, "pool")
            continue
        cout, hw = c
        W, bias = b.recv(9 * cin * cout * 4), b.recv(cout * 4)
        x = b.op([x, W], t(2 * 9 * cin * cout * hw * hw), "conv")
        x = b.op([x, bias], t(cout * hw * hw), "bias")
        x = b.op([x], t(cout * hw * hw), "relu")
        cin = cout
    x = b.op([x], floor, "flatten")
    dims = [(25088, 4096), (4096, 4096), (4096, 1000)]
    for k, (i, o) in enumerate(dims):
        W, bias = b.recv(i * o * 4), b.recv(o * 4)
        x = b.op([x, W], t(2 * i * o), "matmul")
        x = b.op([x, bias], t(o), "bias")
        if k < 2:
            x = b.op([x], t(o), "relu")
    x = b.op([x], floor, "softmax")
    x = b.op([x], floor, "argmax")
    b.op([x], floor, "output")
    return b.finish("vgg16", seed=2, batch=262144, op_dist="lognormal", op_sigma=0.3,
                    recv_sigma=0.2)


def inception3_dag() -> Dag:
    """Preset 4 (seed 3): training graph shaped like Inception v3: a stem of 6
    conv+normalisation units, 11 modules of four parallel branches (1x1 / 1x1 -> 3x3
    factorised / 1x1 -> 5x5 factorised / pool -> 1x1) joined by a concat, a classifier,
    and the mirrored backward pass in which the gradient op of a forward op depends on
    the gradients of its consumers, on the forward op itself and on the parameter recv
    that the forward op reads.  126 convs x (weight, scale, offset) + classifier
    (weight, bias) = 380 recvs."""
    b = _Builder()
    g = _rng(3, _STREAM_STRUCT)
    conv_specs: List[Tuple[float, float]] = []  # (weight bytes, flops) in creation order

    def conv_bn_relu(x: int, cin: int, cout: int, k: int, hw: int) -> int:
        W = b.recv(k * cin * cout * 4)
        ga, be = b.recv(cout * 4), b.recv(cout * 4)
        fl = 2.0 * k * cin * cout * hw * hw
        conv_specs.append((k * cin * cout * 4.0, fl))
        x = _conv_unit(b, x, W, -fl, 5, 5)          # median filled in below (marked negative)
        x = _bn_unit(b, x, ga, be, 10)
        return b.chain([x], [_AUX, _AUX], "relu")

    x = b.op([], _AUX, "input")
    stem = [(3, 32, 9, 149), (32, 32, 9, 147), (32, 64, 9, 147), (64, 80, 1, 73), (80, 192, 9, 71), (192, 192, 9, 35)]
    for (ci, co, k, hw) in stem:
        x = conv_bn_relu(x, ci, co, k, hw)
    x = b.chain([x], [_AUX, _AUX], "pool")
    cin = 192
    for m in range(11):
        hw = 35 if m < 3 else (17 if m < 8 else 8)
        wd = 64 if m < 3 else (192 if m < 8 else 320)
        deep = 4 if m < 10 else 3
        inp = x
        b1 = conv_bn_relu(inp, cin, wd, 1, hw)
        b2 = conv_bn_relu(inp, cin, wd, 1, hw)
        b2 = conv_bn_relu(b2, wd, wd, 3, hw)
        b2 = conv_bn_relu(b2, wd, wd, 3, hw)
        b3 = conv_bn_relu(inp, cin, wd, 1, hw)
        for _ in range(deep):
            b3 = conv_bn_relu(b3, wd, wd, 5 if m < 3 else 7, hw)
        b4 = b.chain([inp], [_AUX, _AUX], "pool")
        b4 = conv_bn_relu(b4, cin, wd, 1, hw)
        b4 = conv_bn_relu(b4, wd, wd, 1, hw)
        x = b.chain([b1, b2, b3, b4], [_AUX, _AUX], "concat")
        cin = 4 * wd
    x = b.chain([x], [_AUX] * 3, "pool")
    Wfc, bfc = b.recv(cin * 1000 * 4), b.recv(1000 * 4)
    x = b.chain([x], [_AUX, _FC, _AUX, _AUX], "fc", feed={1: [Wfc], 3: [bfc]})
    loss = b.chain([x], [_AUX] * 4, "loss")
    del g

    # conv medians in [0.5, 2] ms by FLOPs
    fl = np.array([f for (_, f) in conv_specs])
    med_of = dict(zip(fl.tolist(), _lin_map(fl, 5e-4, 2e-3).tolist()))
    for v in range(len(b.median)):
        if b.median[v] < 0:
            b.median[v] = med_of[-b.median[v]]

    # mirrored backward pass
    n_fwd = len(b.is_recv)
    succ: List[List[int]] = [[] for _ in range(n_fwd)]
    for v in range(n_fwd):
        for p in b.preds[v]:
            succ[p].append(v)
    grad = {}
    for v in range(n_fwd - 1, -1, -1):
        if b.is_recv[v]:
            continue
        preds = [grad[s] for s in succ[v] if s in grad]
        preds.append(v)
        preds += [p for p in b.preds[v] if b.is_recv[p]]
        grad[v] = b.op(preds, 2.0 * b.median[v], "grad_" + b.kind[v])
    assert loss in grad
    return b.finish("inception3", seed=3, batch=65536, op_dist="lognormal", op_sigma=0.4,
                    recv_sigma=0.2)


PRESETS = {
    "tiny": tiny_dag,
    "resnet50": resnet50_dag,
    "vgg16": vgg16_dag,
    "inception3": inception3_dag,
    "stress": stress_dag,
}


def preset(name: str) -> Dag:
    return PRESETS[name]()
