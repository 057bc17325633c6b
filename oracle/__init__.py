"""CPU oracle package (test infrastructure only).

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
anything from here.  The HIP product path never does.
"""
