"""CPU oracle for the batched state-vector path (test infrastructure only).

Nothing in the product package imports this.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg use it.
"""
