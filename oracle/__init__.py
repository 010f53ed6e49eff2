"""CPU oracle for the multi-query attention decode path.  Test infrastructure:
only tests, the smoke check and the benchmark's CPU-baseline leg import it."""
