"""CPU oracle for the MoE feed-forward layer (test infrastructure, not product code)."""
