"""CPU oracle (test infrastructure only): see oracle/deft_oracle.c."""
