"""CPU oracle package: test infrastructure only (tests/, smoke(), bench.py's cpu_baseline)."""
