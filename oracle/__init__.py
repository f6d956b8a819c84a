"""CPU oracle for the HARP rotation path: test infrastructure, never on the product path."""
