"""CPU oracle of the shared-prefix candidate decoding / scoring step.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the CPU-baseline leg
of the benchmark.  The product path never imports it and it imports nothing of the
product."""
