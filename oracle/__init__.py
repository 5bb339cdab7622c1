"""CPU oracle (test infrastructure only; see kfac_oracle.c)."""
