"""CPU oracle for the factored transformer layer.  TEST INFRASTRUCTURE ONLY.

Nothing on the product path may import this package: only tests/, the smoke
check and the benchmark's cpu_baseline leg do.
"""
