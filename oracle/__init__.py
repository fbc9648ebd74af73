"""CPU oracle (test infrastructure).  See jot_oracle.py."""
