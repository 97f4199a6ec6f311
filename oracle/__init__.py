"""CPU oracle (test infrastructure only; see fp6_oracle.c)."""
