"""TicTac scheduling math on MI355X: recv-dependency bitsets, TIC/TAC transfer
priorities and batched makespan / scheduling-efficiency evaluation.

Sub-modules
-----------
workloads : seeded synthetic DAG and timing-sample generators (no scheduling
            arithmetic; shared by the tests of the CPU checker and of the GPU
            path).
binding   : ctypes binding of the C-ABI library (``libtictac.so``) built from
            ``csrc/``; every computation runs in the HIP kernels.
build     : compiles ``csrc/`` for gfx950 with hipcc.

Nothing is imported eagerly so that the generator module can be used on a
machine without the compiled library.
"""

__all__ = ["workloads", "binding", "build"]
