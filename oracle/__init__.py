"""CPU oracle of the MtPC head: test infrastructure only (see mtpc_oracle.py)."""
