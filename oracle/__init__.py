"""CPU oracle for the NeuZip hot path -- test infrastructure only.

Nothing on the product path may import this package; only tests, the smoke
check and the benchmark's CPU-baseline leg do.
"""
