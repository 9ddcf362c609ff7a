"""CPU oracle for one VTC serving step.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 / int64 implementations of what the GPU library computes:

* ``attention``  -- softmax attention over a paged KV cache, written as the
  textbook three-pass definition (the paper, Section 2.1, only says that
  prefill and decode attention over cached tokens exist; it gives no formula).
* ``counters``   -- the virtual-token-counter charge of Algorithm 2 and the
  physical slot index of a paged cache.
* ``scheduler``  -- Algorithm 2 (Virtual Token Counter) on a virtual clock,
  with the length-prediction, general-cost and weighted variants
  (Algorithms 3 and 4, Section 4.3); it produces the ragged batch compositions.
* ``baselines``  -- the evaluation's comparison schedulers FCFS and RPM and
  its service-difference metrics (Section 5.1), in the same simulator.

Nothing here is imported by the product package; only the tests, the smoke
check and the benchmark's CPU-baseline leg may call it.  It shares no code
with the HIP kernels.

Pinning status (see tests/test_oracle_*.py):
  attention  pinned by closed forms, invariants, a library routine and brute force
  counters   pinned by the cost function W = w_p*n_p + w_q*n_q and hand examples
  slots      pinned by brute force
  scheduler  pinned by the paper's lemmas and theorems and hand-traced cases;
             the *composition* of its batches versus the paper's own runs is
             parity unpinned (it depends on policies the paper leaves open).
  baselines  pinned by arrival order, the per-window limit and qualitative
             contrasts with VTC on the paper's synthetic workload shapes
"""
