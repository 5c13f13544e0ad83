"""CPU oracle (test infrastructure only): see fst_oracle.h."""
