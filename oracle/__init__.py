"""fp64 CPU oracle for the Striped / Ring Attention hot path.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product:
it may be imported by the tests, by the smoke check and by the CPU-baseline leg
of the benchmark, and by nothing else.  It shares no code with the HIP library
and never imports it.
"""
