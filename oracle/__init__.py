"""CPU oracle (test infrastructure only; see oracle/vlut_oracle.c)."""
