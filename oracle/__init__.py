"""CPU oracle for paged-KV trajectory attention.  TEST INFRASTRUCTURE ONLY.

Plain, slow, float64 numpy.  It states what the rollout's generation step
computes (paper Sec. 2.1: trajectories alternate LLM generation and tool
calls; Sec. 4.2: a trajectory's KV cache is kept across tool calls and
preemption; Sec. 9: the cache is paged) as the textbook definition of scaled
dot-product attention over a block table, with no tiling, splitting or fusion.

Nothing here is used by the product path: only the tests, the smoke check and
the benchmark's CPU-baseline leg may import this package, and this package
imports nothing from the HIP library or its Python binding.

Pins (all in tests/, runnable without a GPU):
  attention.decode / gather   brute force in pure Python, len=1, identical keys,
                              constant V, block permutation, needle, logit shift
  attention.decode_split      equals attention.decode (combine algebra)
  attention.append            equals repeated decode; chunk-split invariance;
                              dense causal self-attention by brute force
  planner.plan_decode         structural invariants + golden plan written out by hand
  planner.plan_append         structural invariants + brute-force re-derivation
  kv_manager.KVManager        hand-written traces + conservation invariants
  attention.pack / unpack     round trip + hand-written example
"""
