"""Seeded synthetic workloads (shapes and random inputs) shared by the tests, the oracle
runner and the benchmark.  Holds no arithmetic of the method."""
