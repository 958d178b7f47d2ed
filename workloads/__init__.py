"""Seeded synthetic inputs shared by the tests and the benchmark.  Holds none of the method's arithmetic."""
