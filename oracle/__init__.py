"""CPU oracle for the Approximate Random Dropout hot path.

TEST INFRASTRUCTURE ONLY.  Plain, slow NumPy (fp64) written from the paper's
definitions with the dropout mask materialised and applied.  It shares no code
with the HIP library and never imports it.  Only tests, the smoke check and the
``cpu_baseline`` leg of the benchmark may import this package; the product path
never does.
"""
