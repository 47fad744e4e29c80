"""CPU float64 oracle for the Tier-2 attention step (test infrastructure only)."""
