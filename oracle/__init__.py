"""CPU oracle (test infrastructure only; see shplb_oracle.py)."""
