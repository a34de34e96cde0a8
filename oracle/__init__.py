"""CPU oracle for the Gear Training sparse-part step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 restatement of what a Fastgear Worker computes in one
training step (Section 3, sequence steps 4-5) together with the Slowgear
Worker's gradient bookkeeping (Section 1, third point; Section 3, step 6).
Nothing in the product path may import this package; it exists so that the
tests, the smoke check and the benchmark's CPU-baseline leg have something
independent to compare against.  It shares no code with the HIP library.
"""
