"""CPU oracle (test infrastructure only): see kvq_oracle.c for what it computes and cites."""
