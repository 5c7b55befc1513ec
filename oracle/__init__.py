"""CPU oracle: test infrastructure only.

Slow, plain definitions of everything the GPU library computes: the operators
(ops.c, called through ops.py), the tenant forward pass (forward.py), BN
folding (fold.py) and the scheduling layer of the paper (schedule.py).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product library never does.
"""
