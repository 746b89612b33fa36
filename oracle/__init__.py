"""CPU oracle (test infrastructure).  Import only from tests/, smoke() and bench.py's cpu_baseline leg."""
