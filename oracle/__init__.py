"""CPU oracle package: test infrastructure only (see slicemoe_oracle.py)."""
