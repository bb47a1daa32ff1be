"""Seeded synthetic workloads (configs and input generators) used by the tests
and the benchmark.  Holds no arithmetic of the method."""
