"""CPU oracle (test infrastructure only; see pquant_oracle.py)."""
