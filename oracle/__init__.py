"""CPU oracle of the LESS decode path: test infrastructure, never on the product path."""
