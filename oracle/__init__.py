"""CPU oracle for speculative sampling of diffusion chains -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what the HIP library computes, written from the paper and
pinned (tests marked ``not gpu``) to the paper's closed forms and worked examples.  It shares
no code with the library under ``paper_2501_05370_amd/``; only ``tests/``, the smoke check
and the benchmark's CPU-baseline leg may import it.
"""
