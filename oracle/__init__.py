"""CPU oracle of the HDET hot path.  Test infrastructure: only tests, the smoke check and
the benchmark's cpu_baseline leg may import it."""
