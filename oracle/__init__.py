"""CPU oracle for the 1-bit LAMB step: test infrastructure only (tests, smoke check, CPU-baseline
leg of the benchmark).  Never imported by the product package."""
