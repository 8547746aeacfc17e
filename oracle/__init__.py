"""CPU oracle package: test infrastructure only (tests/, the smoke check and the bench's cpu_baseline leg)."""
