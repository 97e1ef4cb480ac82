"""CPU oracle of the TIG batch step: test infrastructure, never part of the product path."""
