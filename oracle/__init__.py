"""CPU oracle for the head-wise joint-attention operator (test infrastructure only)."""
