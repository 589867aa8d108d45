"""CPU oracle of the SRPE serving path.  Test infrastructure: only tests/, the smoke
check and the benchmark's cpu_baseline leg may import this package."""
