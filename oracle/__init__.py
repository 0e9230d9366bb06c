"""Float64 CPU oracle for the CodeNet per-layer coded training step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) imports, calls or links anything in this package; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.  The oracle
shares no code, tables or helpers with the HIP path.
"""
