"""CPU oracle (test infrastructure only): see sfi_oracle.c for what it computes and why."""
