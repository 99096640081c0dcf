"""CPU oracle (test infrastructure only; see gg_oracle.py)."""
