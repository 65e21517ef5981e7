"""fp64 CPU oracle of the batched heterogeneous-adapter LoRA delta (test infrastructure).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
"""
