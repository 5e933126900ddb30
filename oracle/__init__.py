"""CPU oracle for batched candidate-suffix attention (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package;
the HIP product path never does.
"""
