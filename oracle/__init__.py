"""CPU oracle (fp64) for the paged-KV attention path.  Test infrastructure:
only tests/, the smoke check and bench.py's cpu_baseline leg may import it."""
