"""CPU oracle for the local-share collectives and the load balancer.

TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and
the benchmark's CPU-baseline leg import this package; the HIP library and its
Python binding never do, and nothing here imports them.
"""
