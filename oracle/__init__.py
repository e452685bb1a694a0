"""CPU oracle of the token-tree verification step: test infrastructure, not product code."""
