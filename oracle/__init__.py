"""CPU oracle package: test infrastructure only (see hybridkv_oracle.py)."""
