"""CPU oracle (test infrastructure only; see oracle/ckpt_oracle.c)."""
