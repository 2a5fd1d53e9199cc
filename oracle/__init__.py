"""CPU oracle for the two-stage depth-compression DP (test infrastructure).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import this package.  It wraps oracle/dpc_oracle.c (Algorithms 1 and 2 of the
paper plus set recovery) and oracle/dpc_brute.c (exhaustive enumeration of
Eq. 5a, Eq. 6 and Eq. 8 for tiny L) through ctypes, on numpy arrays, and
likewise oracle/dpc_ext_oracle.c / dpc_ext_brute.c (the extended solver of
Appendix B: Algorithms 3 and 4) and oracle/dpc_sweep_oracle.c (importance
normalisation, trade-off curve, latency of a network merged at a given set).
"""
from .api import (  # noqa: F401
    DPC_INF,
    DPC_NOARG,
    stage1,
    stage2,
    relax_row,
    backtrack,
    solve_batch,
    brute_topt,
    brute_objective,
    brute_min_latency_given_A,
    ext_iopt,
    ext_dp,
    ext_backtrack,
    ext_solve_batch,
    brute_ext_objective,
    importance_shift,
    front,
    front_queries,
    chain_latency,
)
