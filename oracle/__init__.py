"""CPU oracle package: test infrastructure only (see finch_oracle.py)."""
