"""CPU oracle (test infrastructure only; see lq_oracle.c)."""
