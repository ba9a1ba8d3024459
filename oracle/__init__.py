"""CPU oracle of the ResQ mixed-precision linear layer (test infrastructure only)."""
