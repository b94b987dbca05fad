"""CPU oracle (test infrastructure only; see vitcop_oracle.py)."""
