"""CPU oracle for the fused generation + scoring stage.  TEST INFRASTRUCTURE ONLY.

Nothing here is part of the product: only the tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it.  It shares no code with the HIP library and never
imports it.  It is written for a reader to check by eye against the method's definition,
not for speed:

* `oracle.transformer` -- what one sample's generation (Section 2.1, "Generation stage":
  prefill, then one token per decoding step until termination) and its inference-stage
  scoring (Section 2.1, "Inference stage": Reference / Reward / Critic forward over the
  prompt and response) compute, in float64 numpy.  Inter-stage fusion (Section 4.1) runs
  sample-level subtasks earlier without changing any sample's result, so the numeric
  oracle is the unfused per-sample definition.
* `oracle.scheduler` -- an integer model of the continuous-batching bookkeeping the fused
  stage performs (admission against the KV budget of Section 4.2's memory constraint,
  page tables, retirement order, scoring-batch formation after the trigger R_t).
* `oracle.gae` -- Generalized Advantage Estimation by its backward recursion (Section 6
  describes the product's variant as one matrix multiply).

Pins: tests/test_oracle_*.py check these against closed forms, brute force on tiny
shapes, invariants, and an independent library implementation of the same decoder.
The paper prints no numeric example for this path, so no value here is pinned to a
printed figure.
"""
