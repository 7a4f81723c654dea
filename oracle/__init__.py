"""CPU oracle package: test infrastructure only (see modse_oracle.py)."""
