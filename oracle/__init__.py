"""CPU oracle (test infrastructure only; see adakv_oracle.py)."""
