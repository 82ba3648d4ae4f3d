"""CPU oracle for the MaxSim hot path (test infrastructure, not the product)."""
