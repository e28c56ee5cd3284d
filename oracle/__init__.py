"""CPU oracle (test infrastructure only).  See made_oracle.py."""
