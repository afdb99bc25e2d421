"""CPU oracle (test infrastructure): see fvdb_oracle.c for what it computes and why."""
