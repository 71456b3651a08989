"""CPU oracle: test infrastructure only (see pac_oracle.c)."""
