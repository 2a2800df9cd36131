"""CPU oracle for on-the-fly operation batching.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the CPU-baseline leg of the benchmark may
import this package; the product path (paper_1705_07860_amd) never does.
"""
