"""Plain CPU oracle for the FineMoE / FineEP MoE-layer hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import, call or
link anything in this directory: only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py do.  The oracle is written from the paper's
definitions in NumPy (fp64 for floating point, int64 for counts), one token or
one expert at a time, with no blocking or fusion, and it shares no code with
the HIP library.

Modules
  router.py  top-K gate (Section 2.1)
  sched.py   load tables, LP optimum (Eq. 1, Eq. 3), canonical replica loads,
             Algorithm 1, permutation indices (Sections 4.1-4.2, 5.1)
  moe.py     expert FFN, dense per-token reference, scheduled path, combine,
             analytic backward (Sections 2.1-2.2, 3)
  placement.py  placement from known loads: greedy replica counts, random
             candidates, Eq. 3 score, choice (Section 5.3)

Every function is pinned by tests/test_oracle_*.py against closed forms,
brute force, the paper's worked example and library routines.  One part is
"parity unpinned" by the paper itself: the exact replica loads x for
restricted placements have no published instance; they are pinned only by the
stated canonical property (lexicographic maximum) checked by exhaustive
enumeration on small instances.  The drawing rule for random placements in
placement.py is a reading of one sentence of Section 5.3 (stated in that
file); what is pinned there is the optimality of the counts, every
candidate's score and the outcome of the Section 6.3 experiment.
"""
