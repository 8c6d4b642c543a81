"""CPU oracle (test infrastructure only; see ffsplit_oracle.py)."""
