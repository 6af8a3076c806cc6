"""CPU oracle package: test infrastructure only (see rpa_oracle.py)."""
