"""fp64 CPU oracle for the attention meta-kernel path (TEST INFRASTRUCTURE ONLY).

This package is the plain, slow definition of what the hot path computes and of
the integer work-unit plan.  It is imported only by the tests, by the smoke check
and by the benchmark's CPU-baseline leg; the product path never routes through
it, and it imports nothing from the HIP path or its Python binding.

Pin status
----------
* ``attention.attention_oracle``   pinned (brute force in pure Python floats,
  closed forms, library dense attention, equivalence identities the paper states).
* ``attention.merge_partials``     pinned (equals whole-row softmax for arbitrary
  key partitions).
* ``planner.plan_oracle``          pinned to the paper's two worked examples and
  to structural invariants; the parameters the paper leaves open (tile sizes,
  tie-breaks, split rule) follow the written plan rules, so beyond those two
  examples the plan is "parity unpinned" by the paper itself.
* ``kv_append.append_kv_oracle``   pinned (round trip against caches generated with
  the rows in place, token-by-token brute force, untouched-byte check, attention
  equivalence, shared prefix blocks never written).
* ``serving.schedule_chunk`` / ``serving.BlockManagerOracle``   pinned (hand-built cases
  for every rule, budget / priority / work-conservation invariants, and a shadow
  cache kept by the test through which every open sequence must read back its own
  tokens after each operation); the rules themselves are readings of prose, so the
  exact tie-breaks are "parity unpinned" by the paper.
* the 2e-2 / 2e-3 tolerance is not from the paper (it states no accuracy).
"""
