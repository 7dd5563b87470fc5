"""CPU oracle of the VER learner step.  TEST INFRASTRUCTURE ONLY.

Plain, slow fp64 numpy/Python written from the paper's description of the
learning phase (section 2.2) and its hyper-parameter table.  Only tests, the
smoke check and the benchmark's CPU-baseline leg may import it.  It shares no
code with the HIP library and never calls it.
"""
