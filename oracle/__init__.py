"""CPU oracle for the binary-coded linear layer (test infrastructure only).

Nothing in the product path may import this package; only tests, the smoke
check and the bench's cpu_baseline leg do.
"""
