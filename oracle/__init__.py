"""CPU oracle (test infrastructure only; see des_oracle.py)."""
