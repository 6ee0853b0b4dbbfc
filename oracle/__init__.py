"""CPU oracle (test infrastructure).  Only tests/, the smoke entry and the
benchmark's cpu_baseline leg may import this package; the library never does."""
