"""CPU fp64 oracle (test infrastructure; never imported by the product path)."""
