"""CPU oracle for the batched discrete Tag roll-out path.

TEST INFRASTRUCTURE ONLY: used by the tests, the smoke check and the benchmark's
CPU-baseline leg.  The product path never imports this package.
"""
