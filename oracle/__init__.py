"""CPU oracle of the AdaPM optimizer step (Alg. 1, Alg. 2, eq. 2-5 of the paper).

TEST INFRASTRUCTURE ONLY.  Plain numpy, fp64 arithmetic, one block at a time,
no blocking / fusion / reordering.  It shares no code with the HIP library and
imports nothing from it.  Only tests, the smoke check and the CPU-baseline leg
of the benchmark may import this package; the product path never does.
"""
