"""CPU oracle for the GoQuant hot path -- test infrastructure only (see goq_oracle.c)."""
