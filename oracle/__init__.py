"""CPU oracle (test infrastructure only; see compactor_oracle.py)."""
