"""CPU oracle (test infrastructure only; see dp_oracle.py)."""
