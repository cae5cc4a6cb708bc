"""CPU oracle for the AMDP pipeline-stage hot path.

TEST INFRASTRUCTURE ONLY. This package is the plain, slow, obviously-correct
definition of what the stage computes, written from the paper (AMDP:
Asynchronous Multi-Directional Pipeline Parallelism): the per-stage schedule
with version tags (Sections 3.1-3.3, Lemma 1 / Lemma B.1, Appendix B.4), the
timed whole-system simulation of Section 3.2 (stage map, FIFO conflicts), the
forward and backward pass of a slice of GPT/BERT transformer blocks (Section
4.1, Table 2), gradient accumulation over a window (Section 3.3) and the Adam
update (Appendix B.1). It shares no code with the HIP library and is imported
only by tests, by the smoke check and by the benchmark's cpu_baseline leg;
the product path never calls it.

Arithmetic is numpy float64 throughout; numpy matmul, scipy's erf and numpy's
elementwise functions are the only library primitives used as steps. A second
tier of the stage's forward and backward (slow_stage.c, loaded by slow.py)
repeats the same definitions as plain C loops over scalars, libm only; the
two tiers are compared with each other in the tests.

Pins (see tests, all runnable without a GPU):
  schedule.generate   Lemma 1 closed form via an independent discrete-event
                      pipeline simulation; the two worked accumulation examples
                      of Section 3.3 / Figure 5; brute-force invariants.
  stage forward       torch.nn.functional fp64 reference ops; causality and
                      padding-independence properties.
  stage backward      central finite differences; torch.autograd fp64.
  scalar-loop tier    the numpy tier (written separately), to 1e-11 of each
                      tensor's largest entry, on tiny shapes and configuration 1.
  accumulate          sum-of-per-minibatch-gradients invariant.
  adam                closed form of the first step; torch.optim.Adam fp64;
                      the bias-correction-free form printed in Appendix B.1.
  system.simulate     serial closed form (one minibatch in flight), the active
                      ratio n/d and the no-bubble statement of Section 3.2, the
                      causal constraints of Appendix B.4 on random cases, a
                      clock-tick re-simulation on tiny cases.
  bf16 rounding       exhaustive comparison with torch's bfloat16 cast on a
                      sweep of bit patterns.
"""
