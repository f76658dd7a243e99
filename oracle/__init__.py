"""CPU oracle (test infrastructure only): see e3_oracle.c and e3_oracle.py."""
