"""CPU oracle (test infrastructure only; see cronus_oracle.py)."""
