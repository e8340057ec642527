"""CPU oracle of the SPA hot path.  Test infrastructure only: imported by tests/, the
smoke check and the benchmark's cpu_baseline leg; never by the product package."""
