"""fp64 CPU checker (test infrastructure only; never imported by the product path)."""
