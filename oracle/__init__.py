"""CPU oracle: test infrastructure only (see seqnet_oracle.py)."""
