"""CPU oracle (test infrastructure; see dppo_oracle.py)."""
