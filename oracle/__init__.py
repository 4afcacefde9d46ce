"""CPU oracle of the FLy verification step (test infrastructure only)."""
