"""CPU oracle for the LAPLEX apply: test infrastructure, never the product path."""
