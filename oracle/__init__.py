"""CPU oracle: test infrastructure only (see vlac_oracle.py)."""
