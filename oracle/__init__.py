"""CPU oracle of the bounded-budget KV step.  Test infrastructure: only tests, the smoke
check and the benchmark's cpu_baseline leg may import it; the product never does."""
