"""CPU oracle for the MTLA path: test infrastructure, never the product path."""
