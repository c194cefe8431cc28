"""CPU oracle (test infrastructure only): see fno_oracle.py."""
