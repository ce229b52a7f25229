"""CPU oracle for the access-pattern hot path.

TEST INFRASTRUCTURE ONLY.  Two independent forms, which the tests require to
agree: `access_pattern` / `programs` (an interpreter of the paper's
access-pattern semantics, numpy) and `brute` (plain C nested loops written from
the paper's element-wise equations).  Only the test suite, the smoke check and
the benchmark's CPU-baseline leg may import this package; the product package
never does.
"""
