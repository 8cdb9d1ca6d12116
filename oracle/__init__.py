"""CPU oracle (test infrastructure only).  See ee_oracle.h."""
