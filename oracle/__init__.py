"""CPU oracle package: test infrastructure only (see rdkv_oracle.py)."""
