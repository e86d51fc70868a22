"""CPU fp64 oracle for sliced, asymmetric-unit causal attention.  TEST INFRASTRUCTURE ONLY.

Everything here is a plain, slow, obviously-correct statement of what the GPU
library must compute; it exists so that tests, the smoke check and the
benchmark's `cpu_baseline` leg can compare against it.  The product path never
imports it, and it imports nothing from the product path.

Modules: attention.py (fp64 causal attention over packed samples, forward and backward, by definition and
table-driven), tables.py (slice table, unit lists, cost model, validation), solver.py (exact min-max partition
by dynamic programming), dag.py (execution timeline of a task graph, 1F1B graph over asymmetric unit lists, memory footprint over the timeline), search.py (the candidate unit counts and the choice among them, composed of the three above).

Parity pins (all in tests/, CPU-only): library cross-check against PyTorch's
fp64 scaled-dot-product attention with autograd, central finite differences,
closed forms (zero queries, single-token samples, key shift), row-sum and
gradient-sum identities, slicing/grouping invariance, brute-force table
enumeration, exhaustive longest paths, the uniform-pipeline closed form and hand-worked fixtures under
tests/golden/.  No function in
this package is "parity unpinned".
"""
