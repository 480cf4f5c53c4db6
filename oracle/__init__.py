"""CPU oracle (test infrastructure).  See ax_oracle.c for what it computes and why."""
