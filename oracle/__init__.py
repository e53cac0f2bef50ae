"""CPU oracle (test infrastructure only; see metok_oracle.py)."""
