"""CPU oracle package: test infrastructure only (see armt_oracle.py)."""
