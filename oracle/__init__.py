"""CPU oracle for the mixed-precision transformer-layer training step.

TEST INFRASTRUCTURE ONLY.  Plain numpy fp64, slow, written from the
definitions; shares no code with the HIP library.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import it; the product path
never does.
"""
