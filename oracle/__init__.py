"""CPU oracle for the quantized GNN layer.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path imports this package; only tests, the smoke check
and the benchmark's cpu_baseline leg do.  It shares no code with the HIP path.
"""
