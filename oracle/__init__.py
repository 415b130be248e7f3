"""CPU oracle (test infrastructure only; see cbm_oracle.py)."""
