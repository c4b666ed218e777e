"""CPU oracle package (test infrastructure; see ess_oracle.py)."""
