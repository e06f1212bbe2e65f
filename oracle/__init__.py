"""float64 CPU oracle of the KV-cache selection pass: test infrastructure only."""
