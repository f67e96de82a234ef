"""CPU oracle: test infrastructure, not part of the product path."""
