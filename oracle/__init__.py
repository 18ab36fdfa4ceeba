"""fp64 CPU oracle for the packed varlen attention + paged KV write path.

TEST INFRASTRUCTURE ONLY.  Nothing under this directory is part of the product path: only
tests/, the smoke check and the benchmark's cpu_baseline leg may import it.  It imports
nothing from the HIP package and shares no code with it.
"""
