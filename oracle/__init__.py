"""CPU oracle (test infrastructure only): see mux_oracle.c and mux_oracle.py."""
