"""CPU oracle for hybrid-batch attention: test infrastructure, not part of the product path."""
