"""Reference oracle: test infrastructure only.

Plain, slow fp64 CPU code that states what the policy-gradient head computes.
Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
it; the product path (the HIP library and its Python binding) never does.
"""
