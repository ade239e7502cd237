"""CPU oracle package: test infrastructure only (see probsparse_oracle.py)."""
