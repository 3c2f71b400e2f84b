"""CPU oracle of the C2R MoE layer: test infrastructure, never imported by the product path."""
