"""CPU oracle: test infrastructure only (see marl_oracle.c for what it follows)."""
