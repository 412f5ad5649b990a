"""CPU float64 oracle for the GSS hot path: test infrastructure only, never imported by the product path."""
