"""CPU oracle for batched hybrid KV-cache restoration.

TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct implementations of
what the restoration hot path computes, written from the paper's statement of
the method.  Only the test-suite, the smoke check and the benchmark's
`cpu_baseline` leg may import this package; the product path never does, and
this package never imports the product path.

Modules
  transformer  decoder forward, split-restore semantics (Sec. 3.1), logits
  planner      batch-aware two-pointer scheduler (Algorithm 1, Sec. 3.3),
               integer cost model, brute-force optimum, L_delta (Sec. 3.1)
  pagetable    lowest-free-first page allocator

Parity pins: every function here is pinned by tests/test_oracle_*.py (closed
forms, invariants, brute force, a torch-CPU library cross-check).  The one
unpinned quantity is the absolute value of cost-model coefficients, which are
hardware measurements ("parity unpinned"); only the plan *given* a cost table
is pinned.
"""
