"""CPU oracle of the pipeline-template planning dynamic program.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
CPU-baseline leg may import this package.  The HIP library and its Python
binding never do, and nothing here imports them.

Contents
  oob_oracle.c   bottom-up int64 implementation of Section 4.1 (the oracle)
  capi.py        ctypes loader / wrapper for the compiled oracle
  topdown.py     second, independent evaluation order: memoised recursion
  brute_force.py exhaustive enumeration of explicit pipelines + closed-form cost
  build.py       compiles oob_oracle.c with gcc
"""
