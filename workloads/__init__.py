"""Seeded synthetic inputs shared by the oracle-side and the library-side of
the tests and the benchmark.  Holds no arithmetic of the method itself."""
