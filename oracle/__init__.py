"""CPU oracle for SCCL-style schedule execution.  TEST INFRASTRUCTURE ONLY.

This package is the slow, plain reference against which the HIP executor is
checked.  It is imported only by the test-suite, by the smoke check and by
the CPU-baseline leg of the benchmark.  It shares no code with the GPU
library and never imports it; the GPU library never imports this package.

Contents (each module cites the passage of the paper it follows):

  topology.py   bandwidth relation B as a list of (edge-set, chunks/round)
                pairs (section 3.2.1), builders for the graphs used here,
                diameter and the ingress bandwidth bound (section 2.4-2.5).
  collective.py relations All/Root/Scattered/Transpose (Table 1) and the
                collectives built from them (Table 2).
  schedule.py   candidate solution (Q, T) of section 3.3 as a small record.
  validate.py   run V_0..V_S, the bandwidth constraint (section 3.3) and the
                contribution-set extension for combining collectives
                (section 3.5).
  generate.py   greedy breadth-first Allgather, ring Allgather, inversion
                (section 3.5), Allreduce = Reducescatter ; Allgather.
  search.py     exhaustive search for the minimal step count on tiny graphs.
  cost.py       (alpha, beta) cost S*alpha + (R/C)*L*beta (section 3.6).
  executor.py   ctypes wrapper around exec.c, the plain schedule executor
                (int32 / fp32 / fp16 with fp32 accumulation).

Parity status: every function above is pinned by tests/test_oracle_*.py to
something other than itself (closed forms, paper tables, brute force); the
one exception is stated where it applies: the bits of an fp sum under a
*different* valid schedule are not comparable (parity unpinned by design;
only the error bound applies).
"""
