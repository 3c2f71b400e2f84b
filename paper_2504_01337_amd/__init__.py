"""MI355X-native hot path of a collaboration-constrained-routing (C2R) MoE layer."""
