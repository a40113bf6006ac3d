"""CPU oracle (test infrastructure only): see mmbp_oracle.c and definition.py."""
