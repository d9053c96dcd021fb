"""Plain CPU oracle (test infrastructure only): `layer` holds the F/B/W pass numerics of a
transformer chunk, `schedule` the building blocks, pass orders and activation-lifetime accounting.
Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this package."""
