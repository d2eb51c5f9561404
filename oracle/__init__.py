"""CPU oracle of the LASAD hot path (fp64, plain C).  Test infrastructure only:
imported by tests, the smoke check and the benchmark's CPU-baseline leg, never
by the HIP package."""
