"""CPU oracle of the M-AVG hot path: test infrastructure, not product code."""
