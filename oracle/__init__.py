"""CPU oracle (test infrastructure). Imported only by tests/, the smoke check and the
benchmark's cpu_baseline leg; never by the product package."""
