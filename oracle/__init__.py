"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

Plain, slow reference implementations written from the paper: the arrangement
enumerator (`oracle.arrangement`) and the fp64 numerical definitions
(`oracle.numeric`, backed by `nt_oracle.c`).  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import this package; the HIP library and its
Python binding never do, and nothing here imports them.
"""
