"""CPU oracle for the low-bit GEMM path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package may import this; only tests, the smoke check and
the benchmark's cpu_baseline leg do.  See gemm_oracle.c (the definition C = A B
on unpacked int8) and bitref.py (the paper's encodings and bitwise product
formulas evaluated word by word on the CPU).
"""
