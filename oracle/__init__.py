"""CPU oracle for the partial-token GRPO loss stage of NAT.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 numpy code written from the
paper's equations; it shares no code with the HIP library and must never be
imported by the product package.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may use it.

Modules
  philox   counter-based generator (Salmon et al., SC'11, Philox4x32-10)
  select   token selection: URS (Sec. 3.1), RPC (Sec. 4, Eq. 7-8, uniform and
           minimum-cutoff variants), deterministic truncation (Sec. 4),
           Horvitz-Thompson weights (Eq. 6, Eq. 9) and mask compaction
  schedule general cut-length distributions q_i and their survival function
           (Sec. 4, Eq. 7-9), Poisson sampling with given inclusion probabilities
           (Sec. 3.1, Eq. 6), prefix packing of the truncated batch (Sec. 4)
  grpo     group-relative advantage (Eq. 2), ratio (Eq. 1), clipped surrogate
           (Eq. 3), sequence-mean objective (Eq. 5) and its gradient w.r.t.
           hidden states and the LM-head matrix (App. A)
  drivers  exhaustive-enumeration and Monte-Carlo expectations of the masked
           estimator (Prop. 1), and the closed-form variances (App. B)

Pinning status: every function here is pinned by tests/test_oracle_*.py
against published known-answer vectors, closed forms printed in the paper,
library routines on textbook special cases, finite differences and
brute-force enumeration.  Nothing is "parity unpinned" except the numerical
values of the paper's accuracy/efficiency tables, which need data, weights
and systems that are not available.
"""
