"""CPU float64 oracle (test infrastructure; never imported by the product path)."""
