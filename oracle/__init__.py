"""CPU oracle (test infrastructure only; see dppo_oracle.py)."""
