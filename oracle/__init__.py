"""CPU oracle (test infrastructure): see gcoo_oracle.c for what each function states."""
