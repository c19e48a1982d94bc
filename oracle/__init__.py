"""CPU oracle (test infrastructure only; see oracle/flowspec_oracle.c)."""
