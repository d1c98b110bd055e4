"""CPU oracle for the checkpoint snapshot path. Test infrastructure only: imported by tests/,
the smoke check and the benchmark's cpu_baseline leg, never by the product package."""
