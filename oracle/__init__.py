"""CPU oracle for the dMoE layer: test infrastructure only, never imported by the product path."""
