"""CPU oracle for Cleave's sub-GEMM hot path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu-baseline leg.  The product package never imports it, and it
imports nothing from the product package.

  planner.py       integer task planner (row/column blocks x K chunks)
  gemm.py          fp64 GEMM, per-task partial blocks, fixed-order aggregation,
                   random-projection check
  cleave_oracle.c  the naive loops behind gemm.py (gcc, OpenMP over rows)

Pins: every function here is checked in tests/test_oracle_*.py against brute
force on tiny shapes, closed forms, exact integer arithmetic and a library
fp64 matmul.  Unpinned by the paper (and so fixed by the test harness, not by
this package): the distribution of heterogeneous tile sizes and of dY.
"""
