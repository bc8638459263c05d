"""CPU oracle for the SLA forward path.  TEST INFRASTRUCTURE ONLY.

A plain, slow float64 numpy statement of what the path computes.  Nothing in
the product (the HIP library and its binding) imports, links or calls anything
here; only tests, the smoke check and the benchmark's CPU-baseline leg do.
"""
