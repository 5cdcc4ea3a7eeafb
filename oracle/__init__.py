"""Oracle package: slow, plain CPU references written from the paper.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only tests, the smoke check and
the benchmark's cpu_baseline leg do.  It shares no code with the GPU path.
"""
