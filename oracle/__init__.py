"""CPU oracle (test infrastructure only): see symi_oracle.py."""
