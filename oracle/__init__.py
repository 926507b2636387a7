"""CPU oracle of the WISV verify round: test infrastructure, never part of the product path."""
