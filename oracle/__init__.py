"""CPU oracle (test infrastructure only; see hero_oracle.py)."""
