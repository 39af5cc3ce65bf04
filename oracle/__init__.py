"""CPU oracle (test infrastructure only): see ff_oracle.c and oracle.py."""
