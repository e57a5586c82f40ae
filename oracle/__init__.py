"""CPU oracle (test infrastructure only). See oracle/patch_oracle.c for what it computes and why."""
