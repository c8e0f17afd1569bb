"""CPU oracle: test infrastructure only (see sdxl_block_oracle.py)."""
