"""Plain fp64 CPU oracle of the sparse-decode hot path.  TEST INFRASTRUCTURE.

This package is the slow, obviously-correct statement of what the path
computes (partition scoring, top-k selection, partition -> page-slot
resolution with the bucketed-LRU budget, attention over the selected pages),
written from the paper.  It shares no code with the HIP path and must never be
imported by the product: only the tests, the smoke check and the benchmark's
CPU-baseline leg may use it.

Floating point is fp64 throughout, fed with the bf16-rounded stored values
converted exactly.  Integer work (indices, slots, masks, LRU state) is exact.
"""
