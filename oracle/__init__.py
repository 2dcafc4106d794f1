"""CPU oracle for type-directed array redistribution (arXiv 2112.01075).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its
Python binding) may import this package; only tests, the smoke check and the
benchmark's CPU-baseline leg do.  It shares no code with the HIP path.
"""
