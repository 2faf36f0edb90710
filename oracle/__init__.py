"""CPU oracle (test infrastructure only; see vabft_oracle.py)."""
