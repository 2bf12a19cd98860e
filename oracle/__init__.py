"""CPU oracle (test infrastructure only): see www_oracle.c.  Import `oracle.oracle` to use it."""
