"""CPU oracle for CTC: test infrastructure only.

Nothing in the product package imports this.  Only tests, the smoke check and
the benchmark's cpu_baseline leg may use it.
"""
