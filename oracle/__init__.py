"""CPU oracle of batch-1 MoE decode with Cache-Prior routing and an LRU expert cache.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; it is
used by tests/, by the smoke check and by the CPU-baseline leg of bench.py.
It is written from the paper's equations in numpy (fp64 for real arithmetic,
explicit fp32 steps where a rounding decides an integer) and shares no code
with the HIP library.
"""
