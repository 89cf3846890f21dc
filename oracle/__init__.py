"""CPU fp64 oracle package: test infrastructure only (tests, smoke check, cpu_baseline)."""
