"""CPU oracle (test infrastructure only).  See pa_oracle.c for what it computes."""
