"""CPU oracle of the replay-evaluation path.  TEST INFRASTRUCTURE: only tests,
the smoke check and the benchmark's CPU-baseline leg import this package."""
