"""CPU oracle (test infrastructure only): see nups_oracle.c and oracle.py."""
