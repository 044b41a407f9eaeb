"""CPU oracle package: test infrastructure only (see basa_oracle.py)."""
