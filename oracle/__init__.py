"""CPU oracle (test infrastructure only; see kan_oracle.py)."""
