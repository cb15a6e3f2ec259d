"""CPU oracle of the Dion step: test infrastructure, never part of the product path."""
