"""CPU oracle of the MoE layer (test infrastructure; see moe_oracle.py)."""
