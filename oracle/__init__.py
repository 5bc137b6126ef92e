"""CPU oracle (test infrastructure only; see layer_oracle.py)."""
