"""CPU oracle for the FLASH-D attention forward pass.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu-baseline leg may import this package; the product (the HIP library and
its Python binding) never does, and this package never imports the product.

  attention.py   whole-tensor fp64 evaluation (C, OpenMP) of the definition,
                 Alg. 1, Alg. 2 and Alg. 3
  recurrence.py  per-row fp64 numpy/Python evaluation from a score vector,
                 with every intermediate w_i and o_i, plus the group-lifted
                 recurrence, the two-state merge and the static skip rule
"""
