"""CPU oracle of the Tsetlin machine hot path.  Test infrastructure only:
imported by tests, the smoke check and the benchmark's cpu_baseline leg."""
