"""CPU oracle for block-sparse attention and its work planner.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path (the HIP library and its Python
binding) imports, calls or links anything in this package; only the tests, the smoke
check and the benchmark's `cpu_baseline` leg do.  The oracle shares no code with the HIP
path: it is written from the paper's definitions in plain numpy, float64.
"""
