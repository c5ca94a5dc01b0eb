"""CPU oracle for the Scaled Outer Product pair search.

TEST INFRASTRUCTURE ONLY: a plain, slow reference written from the paper.  It shares no code with
the HIP path; only tests/, the smoke check and the benchmark's cpu_baseline leg may import it.
"""
