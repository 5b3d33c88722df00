"""CPU oracle (test infrastructure only): see lpq_oracle.c and lpq_oracle.py."""
