"""CPU oracle (test infrastructure only; see locmoe_oracle.py)."""
