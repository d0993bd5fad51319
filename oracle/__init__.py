"""CPU oracle for the MP-LoRA zeroth-order step (test infrastructure only).

Plain NumPy, one perturbed copy at a time, no batching tricks.  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import this package; the product path never does.
"""
