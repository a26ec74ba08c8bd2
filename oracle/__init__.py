"""CPU oracle for the per-token LoRA expert switch (test infrastructure only).

Nothing in the product package imports this; only tests, the smoke check and
the benchmark's cpu_baseline leg do.
"""
