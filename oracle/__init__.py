"""CPU oracle for the rectified sparse-attention layer: test infrastructure only."""
