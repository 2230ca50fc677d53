"""CPU oracle: test infrastructure only (see bcast_oracle.py)."""
